"""Instruction recorder around the CPU oracle (test infrastructure).  The analysis passes of the library count HISA
instructions during a dry run; the independent count comes from here: the oracle's own loops execute the same schedule
with every instruction method wrapped by a counter."""
import contextlib


@contextlib.contextmanager
def recording(o):
    """Yields a dict that fills up while the body runs:
    rotations   key switches of rotations: rotLeft / rotRight by a non-zero amount, and every rotated term of a sum
                that takes its division by P once (those call the oracle's key_switch_acc directly)
    steps       the set of left-rotation amounts they used
    mul_plain   ciphertext x plaintext multiplications;  mul_scalar  ciphertext x integer multiplications
    mul, relinearize, rescale   as named;  add  additions and subtractions of ciphertexts
    min_limbs   the lowest level a result reached
    limb_sum    for rotations, mul, relinearize and rescale: the limbs of the operand, summed over the occurrences"""
    rec = {"rotations": 0, "steps": set(), "mul_plain": 0, "mul_scalar": 0, "mul": 0, "relinearize": 0, "rescale": 0, "add": 0,
           "min_limbs": None, "limb_sum": {"rotations": 0, "mul": 0, "relinearize": 0, "rescale": 0}}
    names = ("rot_left", "mul_plain", "mul_scalar", "mul_int", "mul_no_relin", "relinearize", "div_scalar", "add", "key_switch_acc",
             "mod_down_rescale")
    real = {n: getattr(o, n) for n in names}
    step_of = {}                       # Galois element -> left-rotation amount
    g = 1
    for j in range(o.slots):
        step_of[g] = j
        g = (g * 5) % (2 * o.N)
    nested = [0]                       # rotLeft and relinearize call key_switch_acc themselves: not counted twice

    def low(res):
        l = getattr(res, "limbs", None)
        if l is not None and (rec["min_limbs"] is None or l < rec["min_limbs"]):
            rec["min_limbs"] = l
        return res

    def rot_left(a, steps):            # rotRight goes through here too (it is rotLeft by the complement)
        r = steps % o.slots
        if r:
            rec["rotations"] += 1
            rec["limb_sum"]["rotations"] += a.limbs
            rec["steps"].add(r)
        nested[0] += 1
        try:
            return low(real["rot_left"](a, steps))
        finally:
            nested[0] -= 1

    def relinearize(a):
        rec["relinearize"] += 1
        rec["limb_sum"]["relinearize"] += a.limbs
        nested[0] += 1
        try:
            return low(real["relinearize"](a))
        finally:
            nested[0] -= 1

    def key_switch_acc(d, key_id):
        if not nested[0]:
            if key_id == 0:            # the s^2 key: a relinearisation whose division by P the caller takes itself
                rec["relinearize"] += 1
                rec["limb_sum"]["relinearize"] += d.shape[0]
            else:
                rec["rotations"] += 1
                rec["limb_sum"]["rotations"] += d.shape[0]
                rec["steps"].add(step_of[key_id])
        return real["key_switch_acc"](d, key_id)

    halves = [0]

    def mod_down_rescale(acc, l):      # the division by q_{l-1} P, called once per polynomial of a ciphertext
        halves[0] += 1
        if halves[0] % 2 == 0:
            rec["rescale"] += 1
            rec["limb_sum"]["rescale"] += l
            if rec["min_limbs"] is None or l - 1 < rec["min_limbs"]:
                rec["min_limbs"] = l - 1
        return real["mod_down_rescale"](acc, l)

    def counted(name, key):
        def f(*a, **k):
            rec[key] += 1
            if key in rec["limb_sum"]:
                rec["limb_sum"][key] += a[0].limbs
            return low(real[name](*a, **k))
        return f

    o.rot_left, o.relinearize, o.key_switch_acc = rot_left, relinearize, key_switch_acc
    o.mul_plain = counted("mul_plain", "mul_plain")
    o.mul_scalar = counted("mul_scalar", "mul_scalar")
    o.mul_int = counted("mul_int", "mul_scalar")
    o.mul_no_relin = counted("mul_no_relin", "mul")
    o.div_scalar = counted("div_scalar", "rescale")
    o.add = counted("add", "add")
    o.mod_down_rescale = mod_down_rescale
    try:
        yield rec
    finally:
        for n in names:
            setattr(o, n, real[n])
