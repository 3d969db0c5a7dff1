"""Oracle: the packed homomorphic vector-matrix products (TEST INFRASTRUCTURE).

The algorithms of Sec. 4.1 / App. C (Algorithm 1: activation row times plaintext matrix) and
Sec. 5.1-5.3 (query times K cache, scores times V cache, cache append), written once over a
small operation set so that the same steps run on plain slot vectors (`SlotOps`, no
cryptography) and on oracle ciphertexts (`CkksOps`).
"""
import numpy as np

from .packing import GqaLayout, KvLayout, VmmPlan, _log2


class SlotOps:
    """The CKKS operations of Sec. 2.1 on plain numpy slot vectors."""

    def __init__(self):
        self.rotations = 0
        self.pt_mults = 0
        self.ct_mults = 0

    def add(self, a, b):
        return a + b

    def rotate(self, a, r):
        self.rotations += 1
        return np.roll(a, -r)          # Rot(c, r)[i] = c[i + r]

    def rotate_many(self, a, steps):
        return [self.rotate(a, r) for r in steps]

    def mul_pt(self, a, slots):
        self.pt_mults += 1
        return a * slots

    def mul_ct(self, a, b):
        self.ct_mults += 1
        return a * b

    def relin(self, a):
        return a

    def rescale(self, a):
        return a

    def drop(self, a):
        return a


class CkksOps:
    """The same operations on oracle ciphertexts.  `rotate_many` shares the raised digits of
    the input among its rotations (hoisting)."""

    def __init__(self, ctx, keys, pt_scale=None):
        self.ctx, self.keys = ctx, keys
        self.pt_scale = pt_scale

    def add(self, a, b):
        return self.ctx.ct_add(a, b)

    def rotate(self, a, r):
        return self.ctx.rotate(a, r, self.keys)

    def rotate_many(self, a, steps):
        h = self.ctx.hoist(a)
        return [self.ctx.rotate_hoisted(a, h, r, self.keys) for r in steps]

    def mul_pt(self, a, slots):
        """`slots` is either a slot vector (encoded here at the context scale or pt_scale) or
        an already encoded plaintext."""
        pt = slots if hasattr(slots, "m") else self.ctx.encode(slots, a.level, self.pt_scale)
        return self.ctx.mul_pt(a, pt)

    def mul_ct(self, a, b):
        return self.ctx.mul_ct(a, b)

    def relin(self, a):
        return self.ctx.relinearize(a, self.keys)

    def rescale(self, a):
        return self.ctx.rescale(a)

    def drop(self, a):
        """One level down without touching the message (Sec. 2.1, level drop)."""
        return self.ctx.level_drop(a, a.level - 1)


def _sum(ops, terms):
    acc = terms[0]
    for x in terms[1:]:
        acc = ops.add(acc, x)
    return acc


def vmm_pt(ops, plan: VmmPlan, cx, diagonals):
    """Algorithm 1 (App. C).  cx holds x in the plan's input layout; diagonals[j][k] are the
    weight plaintexts.  Returns y = x W in the plan's output layout (other slots hold partial
    sums until masked, Sec. 4.2), one level lower."""
    # 1. preprocess: interleaved replication
    c = cx
    for r in plan.pre_steps:
        c = ops.add(c, ops.rotate(c, r))
    # 2. baby steps (all rotations of the same ciphertext) and multiply-accumulate
    babies = [c] + ops.rotate_many(c, plan.baby_steps[1:])
    inner = [_sum(ops, [ops.mul_pt(babies[j], diagonals[j][k]) for j in range(plan.r_i)])
             for k in range(plan.r_o)]
    # giant steps, Horner form: one rotation amount reused r_o - 1 times
    acc = inner[plan.r_o - 1]
    for k in range(plan.r_o - 2, -1, -1):
        acc = ops.add(inner[k], ops.rotate(acc, plan.giant_step))
    # 3. reduce inside the ciphertext
    for r in plan.reduce_steps:
        acc = ops.add(acc, ops.rotate(acc, r))
    return ops.rescale(acc)


def vmm_pt_double_hoisted(ctx, keys, plan: VmmPlan, cx, diagonals_ext):
    """Algorithm 1 (App. C) with the baby-step sums kept in the extended basis: the same
    rotations and plaintext products as vmm_pt, but the r_i - 1 hoisted rotations are not
    divided by P one by one; their weighted sums inner_k live on (q_0..q_l, p_0..p_{K-1}) and
    each is divided by P inside the giant step that consumes it.  diagonals_ext[j][k] are the
    weight plaintexts on the extended basis (Context.encode_ext / pt_from_coeffs_ext)."""
    c = cx
    for r in plan.pre_steps:
        c = ctx.ct_add(c, ctx.rotate(c, r, keys))
    hoisted = ctx.hoist(c)
    raised = [ctx.raise_ct(c)] + [ctx.rotate_hoisted_raised(c, hoisted, r, keys) for r in plan.baby_steps[1:]]
    ext = ctx.ext_idx(c.level)
    inner = []
    for k in range(plan.r_o):
        acc = [np.zeros((len(ext), ctx.n), dtype=np.uint64) for _ in range(2)]
        for j in range(plan.r_i):
            ctx.mac_pt_raised(acc, raised[j], diagonals_ext[j][k], c.level)
        inner.append(acc)
    scale = c.scale * diagonals_ext[0][0].scale
    acc = ctx.moddown_ct(inner[plan.r_o - 1], c.level, scale)
    for k in range(plan.r_o - 2, -1, -1):
        acc = ctx.rotate_add_raised(acc, plan.giant_step, keys, inner[k])
    for r in plan.reduce_steps:
        acc = ctx.ct_add(acc, ctx.rotate(acc, r, keys))
    return ctx.rescale(acc)


def vmm_pt_direct_giants(ctx, keys, plan: VmmPlan, cx, diagonals_ext):
    """The same product with the giant steps unrolled: y' = inner_0 + sum_{k>=1} Rot(inner_k, k G)
    (G = plan.giant_step) instead of the nested form Rot(... Rot(inner_{r_o-1}, G) + ..., G).  The
    r_o - 1 rotations no longer depend on each other (they need r_o - 1 keys instead of one); each
    inner_k is rotated where it is, in the extended basis (only its second component is divided by
    P, for the digits of the key switch; ckks.rotate_raised), so that all of them and inner_0 share
    a single final ModDown."""
    c = cx
    for r in plan.pre_steps:
        c = ctx.ct_add(c, ctx.rotate(c, r, keys))
    hoisted = ctx.hoist(c)
    raised = [ctx.raise_ct(c)] + [ctx.rotate_hoisted_raised(c, hoisted, r, keys) for r in plan.baby_steps[1:]]
    ext = ctx.ext_idx(c.level)
    scale = c.scale * diagonals_ext[0][0].scale
    acc = None
    for k in range(plan.r_o):
        inner = [np.zeros((len(ext), ctx.n), dtype=np.uint64) for _ in range(2)]
        for j in range(plan.r_i):
            ctx.mac_pt_raised(inner, raised[j], diagonals_ext[j][k], c.level)
        if k == 0:
            acc = inner
            continue
        R = ctx.rotate_raised(inner, c.level, k * plan.giant_step, keys)
        acc = [ctx.add(acc[0], R[0], ext), ctx.add(acc[1], R[1], ext)]
    y = ctx.moddown_ct(acc, c.level, scale)
    for r in plan.reduce_steps:
        y = ctx.ct_add(y, ctx.rotate(y, r, keys))
    return ctx.rescale(y)


LADDER_GROUP = 3


def ladder_groups(steps):
    """A rotate-and-add ladder c <- c + Rot(c, s_l), l = 0, 1, ..., multiplies by prod_l (1 + Rot_{s_l});
    a run of g consecutive steps equals c + sum over the 2^g - 1 non-empty subsets B of the run of
    Rot(c, sum_{l in B} s_l): rotations of ONE ciphertext.  The ladder is cut into ceil(L / LADDER_GROUP)
    runs of as equal length as possible, the longer ones first (four steps: 2 + 2, six rotations, not
    3 + 1, eight).  Returns the list of rotation amounts of every run (subset with bit pattern b at
    position b - 1)."""
    out, L = [], len(steps)
    runs = -(-L // LADDER_GROUP)
    i = 0
    for r in range(runs):
        g = L // runs + (1 if r < L % runs else 0)
        run = steps[i:i + g]
        i += g
        out.append([sum(s for l, s in enumerate(run) if (b >> l) & 1) for b in range(1, 1 << len(run))])
    return out


def vmm_pt_unrolled(ctx, keys, plan: VmmPlan, cx, diagonals_ext):
    """Algorithm 1 (App. C) computed entirely in the extended basis: the giant steps unrolled as in
    vmm_pt_direct_giants, and the two rotate-and-add ladders (preprocess, reduce) unrolled in runs
    of three steps into hoisted rotations of one ciphertext (ladder_groups).  More rotations (7 per
    run of three instead of 3) but each run has one ModUp, and the whole product one ModDown of
    both components, at its end; second components alone are divided by P where digits are needed."""
    level = cx.level
    ext = ctx.ext_idx(level)
    R = ctx.raise_ct(cx)
    for amounts in ladder_groups(plan.pre_steps):
        R = ctx.rotsum_raised(R, level, amounts, keys)
    # baby steps: hoisted rotations of the (raised) preprocessed ciphertext
    hoisted = ctx.hoist_raised(R, level)
    raised = [R] + [ctx.rotate_raised_hoisted(R, hoisted, level, r, keys) for r in plan.baby_steps[1:]]
    acc = None
    for k in range(plan.r_o):
        inner = [np.zeros((len(ext), ctx.n), dtype=np.uint64) for _ in range(2)]
        for j in range(plan.r_i):
            ctx.mac_pt_raised(inner, raised[j], diagonals_ext[j][k], level)
        if k == 0:
            acc = inner
            continue
        Rk = ctx.rotate_raised(inner, level, k * plan.giant_step, keys)
        acc = [ctx.add(acc[0], Rk[0], ext), ctx.add(acc[1], Rk[1], ext)]
    for amounts in ladder_groups(plan.reduce_steps):
        acc = ctx.rotsum_raised(acc, level, amounts, keys)
    y = ctx.moddown_ct(acc, level, cx.scale * diagonals_ext[0][0].scale)
    return ctx.rescale(y)


def unrolled_steps(plan: VmmPlan):
    """Rotation amounts of vmm_pt_unrolled, in the order they are used."""
    steps = [a for grp in ladder_groups(plan.pre_steps) for a in grp] + list(plan.baby_steps[1:])
    steps += [k * plan.giant_step for k in range(1, plan.r_o)]
    return steps + [a for grp in ladder_groups(plan.reduce_steps) for a in grp]


def direct_giant_steps(plan: VmmPlan):
    """Rotation amounts of vmm_pt_direct_giants: every multiple of the giant step instead of one."""
    steps = list(plan.pre_steps) + list(plan.baby_steps[1:])
    steps += [k * plan.giant_step for k in range(1, plan.r_o)]
    return steps + list(plan.reduce_steps)


def qk_scores(ops, lay: KvLayout, cq, k_cts, masks, replicate=True):
    """Sec. 5.1 with the multi-head layout of Sec. 5.3: scores of one query against the K
    cache.  masks[c] = lay.qk_mask(c) (slot vector or encoded plaintext).  replicate=False: cq is a
    query GROUP (Sec. 5.4: token tau at residue tau, possibly after an inner rotation), nothing is
    replicated, and slot (c, h, tau') of the result is the score of the query at residue tau' against
    key token c t + tau'."""
    for i in range(_log2(lay.t) if replicate else 0):   # replicate q over the t residues
        cq = ops.add(cq, ops.rotate(cq, -(1 << i)))
    acc = None
    for c, kc in enumerate(k_cts):
        p = ops.rescale(ops.relin(ops.mul_ct(cq, kc)))
        for i in range(_log2(lay.E)):                   # sum over the E dims of every head
            p = ops.add(p, ops.rotate(p, (1 << i) * lay.H * lay.t))
        p = ops.mul_pt(p, masks[c])                     # keep copy e = c
        acc = p if acc is None else ops.add(acc, p)
    return ops.rescale(acc)


def qk_unrolled_steps(lay: KvLayout):
    """Rotation amounts of qk_scores_unrolled: the replication ladder of the query as it is, the
    sum over the E dims in runs (ladder_groups)."""
    ladder = [(1 << i) * lay.H * lay.t for i in range(_log2(lay.E))]
    return [-(1 << i) for i in range(_log2(lay.t))] + [a for grp in ladder_groups(ladder) for a in grp]


def qk_scores_unrolled(ctx, keys, lay: KvLayout, cq, k_cts, masks, replicate=True):
    """qk_scores with the sum over the E dims of every head computed in the extended basis: the
    relinearised, rescaled product is raised to (P c0, P c1), every run of the ladder adds the
    hoisted rotations by its subset sums (ckks.rotsum_raised), and one ModDown ends the ladder.
    log2(E) = 7 dependent key switches per key ciphertext become 3 ModUps and 13 inner products.
    masks[c]: the encoded plaintext of lay.qk_mask(c) at the level of the sums."""
    for i in range(_log2(lay.t) if replicate else 0):   # replicate q over the t residues
        cq = ctx.ct_add(cq, ctx.rotate(cq, -(1 << i), keys))
    groups = ladder_groups([(1 << i) * lay.H * lay.t for i in range(_log2(lay.E))])
    acc = None
    for c, kc in enumerate(k_cts):
        p = ctx.rescale(ctx.relinearize(ctx.mul_ct(cq, kc), keys))
        R = ctx.raise_ct(p)
        for amounts in groups:
            R = ctx.rotsum_raised(R, p.level, amounts, keys)
        p = ctx.mul_pt(ctx.moddown_ct(R, p.level, p.scale), masks[c])
        acc = p if acc is None else ctx.ct_add(acc, p)
    return ctx.rescale(acc)


def qk_shared_steps(lay: KvLayout, shared):
    """Rotation amounts of qk_scores_shared: the replication ladder of the query, the runs of the
    per-ciphertext part of the sum over the dims (strides shared * 2^i blocks), the shared - 1 shared rotations."""
    Ht = lay.H * lay.t
    ladder = [(shared << i) * Ht for i in range(_log2(lay.E // shared))]
    steps = [-(1 << i) for i in range(_log2(lay.t))] + [a for grp in ladder_groups(ladder) for a in grp]
    return steps + [k * Ht for k in range(1, shared)]


def qk_scores_shared_ops(ops, lay: KvLayout, cq, k_cts, masks, shared, replicate=True):
    """q K^T with the mask applied BEFORE the last `shared` terms of the sum over the dims (Sec. 5.1 sums
    over all E copies of every key ciphertext's product and then keeps copy e = c).  With E = shared * E2
    and B = H t slots per copy,
        mask_c * sum_{k < E} Rot(P_c, k B) = sum_{k1 < shared} Rot( mask_{c + k1} * T_c, k1 B ),
        T_c = sum_{k2 < E2} Rot(P_c, k2 shared B),
    because Rot(a b) = Rot(a) Rot(b) and a right rotation of mask_c by k1 copies is mask_{c + k1}.  Summed
    over c, the outer rotations act on A_k1 = sum_c mask_{c + k1} T_c: shared - 1 rotations for the whole
    cache instead of log2(shared) per key ciphertext.  masks[b] = lay.qk_mask(b) for b < E.  The same
    scores as qk_scores; shared = 1 is qk_scores itself."""
    B = lay.H * lay.t
    for i in range(_log2(lay.t) if replicate else 0):
        cq = ops.add(cq, ops.rotate(cq, -(1 << i)))
    T = []
    for kc in k_cts:
        p = ops.rescale(ops.relin(ops.mul_ct(cq, kc)))
        for i in range(_log2(lay.E // shared)):
            p = ops.add(p, ops.rotate(p, (shared << i) * B))
        T.append(p)
    acc = None
    for k1 in range(shared):
        a = _sum(ops, [ops.mul_pt(T[c], masks[(c + k1) % lay.E]) for c in range(len(T))])
        a = a if k1 == 0 else ops.rotate(a, k1 * B)
        acc = a if acc is None else ops.add(acc, a)
    return ops.rescale(acc)


def qk_scores_shared(ctx, keys, lay: KvLayout, cq, k_cts, masks, shared, replicate=True):
    """qk_scores_shared_ops in the extended basis: the per-ciphertext part of the sum as in
    qk_scores_unrolled (runs of hoisted rotations, one ModDown per key ciphertext), then
    P A_0 + sum_k1 RotRaised(A_k1, k1 B) and one ModDown for the whole cache.  masks[b]: the encoded
    plaintext of lay.qk_mask(b) at the level of the sums, b < E."""
    B = lay.H * lay.t
    for i in range(_log2(lay.t) if replicate else 0):
        cq = ctx.ct_add(cq, ctx.rotate(cq, -(1 << i), keys))
    groups = ladder_groups([(shared << i) * B for i in range(_log2(lay.E // shared))])
    T = []
    for kc in k_cts:
        p = ctx.rescale(ctx.relinearize(ctx.mul_ct(cq, kc), keys))
        if groups:
            R = ctx.raise_ct(p)
            for amounts in groups:
                R = ctx.rotsum_raised(R, p.level, amounts, keys)
            p = ctx.moddown_ct(R, p.level, p.scale)
        T.append(p)
    lv = T[0].level
    ext = ctx.ext_idx(lv)
    acc = None
    for k1 in range(shared):
        a = None
        for c in range(len(T)):
            t = ctx.mul_pt(T[c], masks[(c + k1) % lay.E])
            a = t if a is None else ctx.ct_add(a, t)
        if k1 == 0:
            acc, scale = ctx.raise_ct(a), a.scale
        else:
            R = ctx.rotate_hoisted_raised(a, ctx.hoist(a), k1 * B, keys)
            acc = [ctx.add(acc[0], R[0], ext), ctx.add(acc[1], R[1], ext)]
    return ctx.rescale(ctx.moddown_ct(acc, lv, scale))


def qk_scores_indexed(ops, lay: KvLayout, cq, x_cts, replicate=True, sv=None):
    """q K^T from the key index.  Sec. 5.1: scores = sum_c mask_c sum_k Rot(q . K_c, k B) (B = H t).  With
    Rot(a b) = Rot(a) Rot(b):  = sum_k Rot(q, k B) . D_k,  D_k = sum_c mask_c Rot(K_c, k B), which depends on the
    cache only: copy c of D_k holds dim (c + k) mod E of key group c.  That is a product of the diagonal form of
    Sec. 5.2 (scores V) with q in the place of the scores and the D_k in the place of the V ciphertexts, so its
    baby-step / giant-step schedule is used as it is: x_cts[g r_i + j] = Rot(D_{g r_i + j}, -g r_i B)
    (lay.pack_k_index), scores = sum_g Rot( sum_j Rot(q, j B) (x) x_cts[g r_i + j], g r_i B ), one
    relinearisation per giant-step group, no mask afterwards (one level less than qk_scores), no sum over the
    residues.  `sv` = the scores-times-V routine to run (score_times_v, or the extended-basis one bound to its
    context and keys)."""
    for i in range(_log2(lay.t) if replicate else 0):   # replicate q over the t residues
        cq = ops.add(cq, ops.rotate(cq, -(1 << i)))
    if sv is not None:
        return sv(cq, x_cts)
    return score_times_v(ops, lay, cq, x_cts, reduce=False)


def score_times_v(ops, lay: KvLayout, cs, v_cts, reduce=True):
    """Sec. 5.2/5.3: Att[h, e] = sum_n s[h, n] V[n, h, e]; result at (e, h, 0), the input
    layout of the next plaintext product (other residues hold partial sums).  reduce=False
    (Sec. 5.4, scores of a query group): the residues are not summed, slot (e, h, tau) holds
    sum_c s[c, h, tau] V[c t + tau, h, e], the contribution of the keys at residue tau to the query
    whose scores sit at residue tau."""
    babies = [cs] + ops.rotate_many(cs, [j * lay.H * lay.t for j in range(1, lay.r_i)])
    inner = []
    for g in range(lay.r_o):
        terms = [ops.mul_ct(babies[j], v_cts[g * lay.r_i + j]) for j in range(lay.r_i)]
        inner.append(ops.relin(_sum(ops, terms)))
    acc = inner[lay.r_o - 1]
    for g in range(lay.r_o - 2, -1, -1):
        acc = ops.add(inner[g], ops.rotate(acc, lay.r_i * lay.H * lay.t))
    acc = ops.rescale(acc)
    for l in range(_log2(lay.t) if reduce else 0):
        acc = ops.add(acc, ops.rotate(acc, 1 << l))
    return acc


def sv_unrolled_steps(lay: KvLayout):
    """Rotation amounts of score_times_v_unrolled: baby steps, every multiple of the giant step, the
    runs of the residue ladder."""
    Ht = lay.H * lay.t
    steps = [j * Ht for j in range(1, lay.r_i)] + [g * lay.r_i * Ht for g in range(1, lay.r_o)]
    return steps + [a for grp in ladder_groups([1 << l for l in range(_log2(lay.t))]) for a in grp]


def score_times_v_unrolled(ctx, keys, lay: KvLayout, cs, v_cts, reduce=True):
    """score_times_v without dependent rotations after the products: the giant steps unrolled
    (sum_g Rot(inner_g, g G), each rotation left in the extended basis next to P inner_0) and the
    reduce ladder over the residues run there too, in runs of hoisted rotations (ckks.rotsum_raised),
    before one ModDown and the rescale (the ladder form rescales first and reduces one level lower;
    the message is the same).  reduce=False: no ladder over the residues (see score_times_v)."""
    Ht, lv = lay.H * lay.t, cs.level
    ext = ctx.ext_idx(lv)
    h = ctx.hoist(cs)
    babies = [cs] + [ctx.rotate_hoisted(cs, h, j * Ht, keys) for j in range(1, lay.r_i)]
    inner = []
    for g in range(lay.r_o):
        acc = None
        for j in range(lay.r_i):
            t = ctx.mul_ct(babies[j], v_cts[g * lay.r_i + j])
            acc = t if acc is None else ctx.ct_add(acc, t)
        inner.append(ctx.relinearize(acc, keys))
    T = ctx.raise_ct(inner[0])
    for g in range(1, lay.r_o):
        R = ctx.rotate_hoisted_raised(inner[g], ctx.hoist(inner[g]), g * lay.r_i * Ht, keys)
        T = [ctx.add(T[0], R[0], ext), ctx.add(T[1], R[1], ext)]
    for amounts in ladder_groups([1 << l for l in range(_log2(lay.t) if reduce else 0)]):
        T = ctx.rotsum_raised(T, lv, amounts, keys)
    return ctx.rescale(ctx.moddown_ct(T, lv, inner[0].scale))


def masked_two_rotations(ops, c, plaintexts, up, down):
    """c p0 + Rot(c p2, up) + Rot(c p1, down), then the rescale: three plaintext products, two
    rotations, one level."""
    p0, p1, p2 = plaintexts
    y = ops.mul_pt(c, p0)
    y = ops.add(y, ops.rotate(ops.mul_pt(c, p2), up))
    y = ops.add(y, ops.rotate(ops.mul_pt(c, p1), down))
    return ops.rescale(y)


def rope(ops, lay: KvLayout, c, plaintexts):
    """App. D: c p0 + Rot(c p2, +H t) + Rot(c p1, -H t), then the rescale; three plaintext products,
    two rotations, one level.  `plaintexts` = lay.rope_plaintexts(n, tau) (slot vectors or encoded
    plaintexts); slots outside the valid ones come out zero whatever they held."""
    return masked_two_rotations(ops, c, plaintexts, lay.rope_step, -lay.rope_step)


def inner_rotate(ops, lay: KvLayout, c, delta, plaintexts):
    """Sec. 5.4, the 'inner rotations' of the prompt-phase Q K^T: residue tau of every block moves to
    residue (tau + delta) mod t, so that a query group meets the keys of other residues.
    `plaintexts` = lay.inner_rotation_plaintexts(delta)."""
    up, down = lay.inner_rotation_steps(delta)
    return masked_two_rotations(ops, c, plaintexts, up, down)


def _index_append(ops, lay, x_cts, ck_new, x_masks):
    """x_cts[g r_i + j] += mask * Rot(ck_new, j B): the baby rotations of the new key(s) are rotations of one
    ciphertext (hoisted); x_masks[k] = lay.k_index_append_mask(k, n) or its group form."""
    rotated = [ck_new] + ops.rotate_many(ck_new, [j * lay.H * lay.t for j in range(1, lay.r_i)])
    for k in range(lay.E):
        xnew = ops.rescale(ops.mul_pt(rotated[k % lay.r_i], x_masks[k]))
        x_cts[k] = xnew if x_cts[k] is None else ops.add(x_cts[k], xnew)


def kv_append(ops, lay: KvLayout, k_cts, v_cts, n, ck_new, cv_new, k_mask, v_masks, x_cts=None, x_masks=None):
    """Append token n = c*t + tau (Sec. 5.1 'K Cache Update', Sec. 5.2 'V Cache Update').
    ck_new / cv_new carry the new vectors at residue tau (other slots may hold partial sums);
    k_mask = lay.residue_mask(tau), v_masks[k] = lay.v_append_mask(k, n).  Masking costs the
    level the paper fuses with RoPE; the cache ciphertexts live one level below the inputs."""
    c = n // lay.t
    knew = ops.rescale(ops.mul_pt(ck_new, k_mask))
    if c == len(k_cts):
        k_cts.append(knew)
    else:
        k_cts[c] = ops.add(k_cts[c], knew)
    # the shifts are rotations of one ciphertext: they share its raised digits (hoisting)
    shifted = [cv_new] + ops.rotate_many(cv_new, [-(g * lay.r_i * lay.H * lay.t) for g in range(1, lay.r_o)])
    for k in range(lay.E):
        vnew = ops.rescale(ops.mul_pt(shifted[k // lay.r_i], v_masks[k]))
        v_cts[k] = vnew if v_cts[k] is None else ops.add(v_cts[k], vnew)
    if x_cts is not None:
        _index_append(ops, lay, x_cts, ck_new, x_masks)


def kv_append_group(ops, lay: KvLayout, k_cts, v_cts, c, ck_grp, cv_grp, k_mask, v_masks, x_cts=None, x_masks=None):
    """Sec. 5.4, cache generation in the prompt phase: the t tokens c*t .. c*t + t-1 at once.
    ck_grp / cv_grp hold token c*t + tau at residue tau of every (e, h) block, which is already
    the layout of K ciphertext c; k_mask is all ones (the product only keeps levels and scales
    equal to the one-token update), v_masks[k] = lay.v_append_group_mask(k, c)."""
    assert c == len(k_cts)
    k_cts.append(ops.rescale(ops.mul_pt(ck_grp, k_mask)))
    shifted = [cv_grp] + ops.rotate_many(cv_grp, [-(g * lay.r_i * lay.H * lay.t) for g in range(1, lay.r_o)])
    for k in range(lay.E):
        vnew = ops.rescale(ops.mul_pt(shifted[k // lay.r_i], v_masks[k]))
        v_cts[k] = vnew if v_cts[k] is None else ops.add(v_cts[k], vnew)
    if x_cts is not None:
        _index_append(ops, lay, x_cts, ck_grp, x_masks)


def gqa_qk_scores(ops, glay: GqaLayout, cq, k_cts, masks, rot_plaintexts, qk=None):
    """q K^T of one token against a cache that stores every KV head once (packing.GqaLayout).  cq: the query
    at (e, h, 0) of the H-head layout, one level above the cache.  It is replicated over its t residues
    (Sec. 5.1 step 1), then for every pass delta moved by the inner rotation of delta t residues (Sec. 5.4;
    pass 0 only drops the level) and multiplied into the cache WITHOUT further replication (qk_scores with
    replicate=False).  rot_plaintexts[delta] = glay.kv.inner_rotation_plaintexts(delta t) (slot vectors or
    encoded plaintexts), masks[c] as for qk_scores on glay.kv.  Returns the G score ciphertexts, two levels
    below the cache.  `qk` = the q K^T routine to run per pass (default: the printed order)."""
    for i in range(_log2(glay.t)):
        cq = ops.add(cq, ops.rotate(cq, -(1 << i)))
    outs = []
    for delta in range(glay.G):
        x = ops.drop(cq) if delta == 0 else inner_rotate(ops, glay.kv, cq, glay.inner_delta(delta), rot_plaintexts[delta])
        outs.append(qk(x) if qk is not None else qk_scores(ops, glay.kv, x, k_cts, masks, replicate=False))
    return outs


def gqa_score_times_v(ops, glay: GqaLayout, cs_list, v_cts, rot_plaintexts, sv=None):
    """scores V for the same layout.  cs_list[delta]: the scores of pass delta (the layout gqa_qk_scores
    writes, GqaLayout.pack_scores), at the cache level.  Every pass meets V without the sum over the residues
    (score_times_v with reduce=False), is moved back by the inner rotation of (G - delta) t residues (pass 0
    only drops the level), the passes are added, and the t residues of a query head's run are summed by
    log2(t) rotate-and-add steps.  Result: Att[h, e] at (e, h, 0) of the H-head layout, two levels below the
    cache.  rot_plaintexts[b] = glay.kv.inner_rotation_plaintexts(b t)."""
    acc = None
    for delta in range(glay.G):
        part = sv(cs_list[delta]) if sv is not None else score_times_v(ops, glay.kv, cs_list[delta], v_cts, reduce=False)
        back = (glay.G - delta) % glay.G
        part = ops.drop(part) if back == 0 else inner_rotate(ops, glay.kv, part, glay.inner_delta(back), rot_plaintexts[back])
        acc = part if acc is None else ops.add(acc, part)
    for l in range(_log2(glay.t)):
        acc = ops.add(acc, ops.rotate(acc, 1 << l))
    return acc
