"""Oracle: slot layouts of interleaved replicated packing (TEST INFRASTRUCTURE).

Everything here is about WHERE numbers sit in the S slots of a ciphertext: the activation
layouts and the weight-diagonal plaintexts of the packed vector-matrix product (Sec. 4.1,
App. C / Algorithm 1) and the K-cache, V-cache, query, score and mask layouts of the
attention products (Sec. 5.1-5.3).  No cryptography.

Notation (the paper's, with S for its slot count N): d = length of the shorter vector,
t = S/d its interleave interval; alpha = aspect ratio; t' = S/(alpha d) the interval of the
longer vector.  A slot index is written i = b*t + r (block b, residue r), and for the longer
vector r = s*t' + r'.

Readings taken where the printed algorithm and the text disagree:
  * the preprocess rotation is 2^i (t-1) slots (the toy example of Sec. 4.1 needs a rotation
    by t-1 = 1 to reach [a0,a1,a1,a2,...]; a rotation by d-1 does not give it);
  * rotation amounts printed as j t' and t r_i count blocks; in slots they are j t' t and
    r_i t' t, and r_o = d / (t' r_i), the only choice with r_i r_o t' = d;
  * the weight plaintexts are built by pushing index labels through the same rotations
    instead of using the printed closed forms;
  * token-batched products (Sec. 5.4, the prompt phase): the text only says that a ciphertext
    "holds t tokens without preprocessing".  Read as: residue tau of block b holds element b of
    token tau, the preprocess and reduce steps disappear, and the product is the diagonal
    method over all d diagonals with every rotation a whole number of blocks (baby step j t,
    giant step r_i t), each weight diagonal repeated over the residues.  Square shapes only: a
    wider or taller matrix is a set of square ones.
"""
from dataclasses import dataclass
from typing import List

import numpy as np


def _log2(x):
    assert x > 0 and x & (x - 1) == 0, x
    return x.bit_length() - 1


@dataclass
class VmmPlan:
    S: int
    d: int          # shorter dimension
    alpha: int
    mode: str       # "square" (d->d), "expand" (d -> alpha d), "contract" (alpha d -> d)
    r_i: int
    tau: int = 0    # residue the valid output lands on (0 unless preparing a cache append)
    tokens: bool = False   # token-batched: residue tau holds token tau, t tokens per ciphertext

    def __post_init__(self):
        self.t = self.S // self.d
        self.tp = self.S // (self.alpha * self.d)
        assert self.t * self.d == self.S and self.tp * self.alpha * self.d == self.S
        assert self.mode in ("square", "expand", "contract")
        assert (self.alpha == 1) == (self.mode == "square")
        self.t1, self.t2 = (self.tp, self.t) if self.mode == "contract" else (self.t, self.tp)
        if self.tokens:
            # nothing is replicated or summed inside a block; rotations move whole blocks
            assert self.mode == "square"
            self.tp = self.t1 = self.t2 = 1
        self.M = self.d // self.tp                      # number of diagonals
        assert self.M >= 1 and self.M % self.r_i == 0
        self.r_o = self.M // self.r_i
        assert 0 <= self.tau < self.t2
        self.d_in = self.d * (self.alpha if self.mode == "contract" else 1)
        self.d_out = self.d * (self.alpha if self.mode == "expand" else 1)

    # rotation amounts, in slots
    @property
    def pre_steps(self) -> List[int]:
        return [(1 << i) * (self.t - 1) for i in range(_log2(self.t1))]

    @property
    def baby_steps(self) -> List[int]:
        return [j * self.tp * self.t for j in range(self.r_i)]

    @property
    def giant_step(self) -> int:
        return self.r_i * self.tp * self.t

    @property
    def reduce_steps(self) -> List[int]:
        """2^l to the left, or to the right where bit l of tau is set: the block of t2 slots
        then sums into residue tau instead of 0 (the 'customizable' packing of Sec. 5.1)."""
        return [-(1 << l) if (self.tau >> l) & 1 else (1 << l) for l in range(_log2(self.t2))]

    @property
    def n_rotations(self):
        return _log2(self.t1) + (self.r_i - 1) + (self.r_o - 1) + _log2(self.t2)

    def all_steps(self):
        s = self.pre_steps + self.baby_steps[1:] + self.reduce_steps
        if self.r_o > 1:
            s.append(self.giant_step)
        return s

    # layouts ---------------------------------------------------------------------------
    def in_slot(self, a):
        """Slot of input element a."""
        if self.mode == "contract":
            return (a % self.d) * self.t + (a // self.d) * self.tp
        return a * self.t

    def out_slot(self, c):
        if self.mode == "expand":
            return (c % self.d) * self.t + (c // self.d) * self.tp + self.tau
        return c * self.t + self.tau

    def pack_input(self, x):
        v = np.zeros(self.S)
        v[[self.in_slot(a) for a in range(self.d_in)]] = x
        return v

    def unpack_output(self, slots):
        return np.asarray(slots)[[self.out_slot(c) for c in range(self.d_out)]]

    def out_mask(self):
        m = np.zeros(self.S)
        m[[self.out_slot(c) for c in range(self.d_out)]] = 1.0
        return m

    def pack_tokens(self, X):
        """Token-batched input: X[tau, b] at slot b*t + tau."""
        X = np.asarray(X)
        assert self.tokens and X.shape == (self.t, self.d)
        return X.T.reshape(-1).copy()

    def unpack_tokens(self, slots):
        return np.asarray(slots).reshape(self.d, self.t).T

    def block_col(self):
        """Output index owned by each block of t2 consecutive slots (of t slots when
        token-batched)."""
        if self.tokens:
            return np.arange(self.d)
        B = np.arange(self.S // self.t2)
        if self.mode == "expand":
            return B // self.alpha + (B % self.alpha) * self.d
        return B

    def source_labels(self):
        """Input index held by every slot after the preprocess step (labels pushed through
        the same rotate-and-add; two labelled slots never meet)."""
        if self.tokens:
            return np.arange(self.S) // self.t
        lab = np.full(self.S, -1, dtype=np.int64)
        for a in range(self.d_in):
            lab[self.in_slot(a)] = a
        for r in self.pre_steps:
            rot = np.roll(lab, -r)
            assert not np.any((lab >= 0) & (rot >= 0))
            lab = np.where(rot >= 0, rot, lab)
        assert np.all(lab >= 0)
        return lab

    def diagonals(self, W):
        """Slot vectors p[j][k] of the weight plaintexts: slot i' of Rot(c', baby_j) holds
        input index row; its product ends, after k giant rotations and the reduce step, in the
        block that owns output index col."""
        W = np.asarray(W)
        assert W.shape == (self.d_in, self.d_out)
        lab, col_of_block, S = self.source_labels(), self.block_col(), self.S
        i = np.arange(S)
        out = [[None] * self.r_o for _ in range(self.r_i)]
        for j in range(self.r_i):
            row = np.roll(lab, -self.baby_steps[j])
            for k in range(self.r_o):
                col = col_of_block[((i - k * self.giant_step) % S) // (self.t if self.tokens else self.t2)]
                out[j][k] = W[row, col]
        return out


def default_r_i(M):
    """Baby-step count: the power of two at or just above sqrt(M)."""
    return 1 << ((_log2(M) + 1) // 2)


def make_plan(S, d_in, d_out, r_i=None, tau=0, tokens=False):
    if tokens:
        assert d_in == d_out
        # twice the square-root rule: the baby steps are hoisted rotations of one ciphertext, several times cheaper
        # than the giant steps, each of which raises a ciphertext of its own
        return VmmPlan(S, d_in, 1, "square", min(d_in, 2 * default_r_i(d_in)) if r_i is None else r_i, 0, True)
    if d_in == d_out:
        d, alpha, mode = d_in, 1, "square"
    elif d_out > d_in:
        d, alpha, mode = d_in, d_out // d_in, "expand"
    else:
        d, alpha, mode = d_out, d_in // d_out, "contract"
    M = d // (S // (alpha * d))
    return VmmPlan(S, d, alpha, mode, default_r_i(M) if r_i is None else r_i, tau)


# ---- attention layouts (Sec. 5) ------------------------------------------------------------
@dataclass
class KvLayout:
    """Slot (e, h, tau) := (e*H + h)*t + tau with t = S/(H*E): head-interleaved blocks of t
    (Sec. 5.3).  A query / key / value vector of the current token has element [h, e] at
    (e, h, tau); K ciphertext c holds token c*t + tau at residue tau; the score ciphertext
    holds token c*t + tau of head h at (c, h, tau), so it has room for E*t = S/H tokens;
    V ciphertext k holds V[((e + k) mod E)*t + r, h, e] at (e, h, r), stored rotated right by
    the giant step of its BSGS group.
    A head count that is not a power of two (GPT2-base: 12 heads of 64 dims, Table 3) is padded to the
    next one, as the paper pads that model's width 768 to 1024 (Table 4): H becomes the padded count (the
    stride of the layout), `heads` keeps the real one; the padding heads hold zeros, vectors and scores
    are exchanged for the real heads only."""
    S: int
    H: int
    E: int
    r_i: int = 0    # baby steps of the score-times-V product; 0 -> E (no giant steps)

    def __post_init__(self):
        self.heads = self.H
        self.H = 1 << (self.H - 1).bit_length()
        self.t = self.S // (self.H * self.E)
        assert self.t * self.H * self.E == self.S
        self.r_i = self.r_i or self.E
        assert self.E % self.r_i == 0
        self.r_o = self.E // self.r_i
        self.capacity = self.E * self.t

    def slot(self, e, h, tau):
        return (e * self.H + h) * self.t + tau

    def pack_vec(self, v, tau=0):
        """v[h, e] at (e, h, tau), zero elsewhere."""
        out = np.zeros(self.S)
        for h in range(self.heads):
            for e in range(self.E):
                out[self.slot(e, h, tau)] = v[h, e]
        return out

    def unpack_vec(self, slots, tau=0):
        return np.array([[slots[self.slot(e, h, tau)] for e in range(self.E)]
                         for h in range(self.heads)])

    # ---- rotary position embedding with the extraction fused (Sec. 4.2, App. D) --------------
    # The embedding turns the pair of dims (2m, 2m+1) of every head by the angle
    # theta(m, n) = n * base^(-2m/E) of token n.  In this layout the two dims of a pair sit one
    # block row apart, H*t slots (the appendix writes the single-head case, where that is one block
    # of t slots, as "rotate by 1").  Reading of the rotation signs (the printed ones do not fit the
    # left-rotation convention of Sec. 2.1): the odd dim comes to the even one by a LEFT rotation of
    # the product with p2, the even dim to the odd one by a RIGHT rotation of the product with p1.
    def rope_angle(self, e, n, base=10000.0):
        return n * base ** (-2.0 * (e // 2) / self.E)

    def rope_plaintexts(self, n, tau=0, base=10000.0):
        """(p0, p1, p2): cos on the valid slots; sin on the valid slots of even dims; -sin on those
        of odd dims.  Every other slot is zero, which is the extraction."""
        p0, p1, p2 = np.zeros(self.S), np.zeros(self.S), np.zeros(self.S)
        for e in range(self.E):
            th = self.rope_angle(e, n, base)
            for h in range(self.H):
                i = self.slot(e, h, tau)
                p0[i] = np.cos(th)
                if e % 2 == 0:
                    p1[i] = np.sin(th)
                else:
                    p2[i] = -np.sin(th)
        return p0, p1, p2

    def rope_plaintexts_group(self, c, base=10000.0):
        """The same for a ciphertext that holds the t tokens c*t .. c*t + t-1, token c*t + tau at
        residue tau (the prompt phase, Sec. 5.4): every residue gets the angles of its own token."""
        ps = [self.rope_plaintexts(c * self.t + tau, tau, base) for tau in range(self.t)]
        return tuple(sum(p[i] for p in ps) for i in range(3))

    @property
    def rope_step(self):
        return self.H * self.t

    # ---- inner rotation (Sec. 5.4): residues moved cyclically inside every block of t ---------------
    # InnerRot_delta(x)[b, tau'] = x[b, (tau' - delta) mod t].  A slot rotation by -delta does that for
    # the residues that do not wrap (tau < t - delta before the move); those that wrap come from a
    # rotation by t - delta.  Masking BEFORE the rotations (zero plaintext for the unrotated term)
    # gives it the shape of the rotary embedding: two rotations, one level.
    def inner_rotation_steps(self, delta):
        assert 0 < delta < self.t
        return [-delta, self.t - delta]

    def inner_rotation_plaintexts(self, delta):
        """(p0, p1, p2) for vmm.masked_two_rotations with steps (up, down) = inner_rotation_steps:
        p0 = 0; p2 = residues below t - delta (moved by -delta); p1 = the others (moved by t - delta)."""
        r = np.arange(self.S) % self.t
        return np.zeros(self.S), (r >= self.t - delta).astype(float), (r < self.t - delta).astype(float)

    def pack_k(self, K, c):
        """K[token, h, e] -> slots of K ciphertext c (tokens past the end are zero)."""
        out = np.zeros(self.S)
        for tau in range(self.t):
            n = c * self.t + tau
            if n < K.shape[0]:
                out += self.pack_vec(K[n], tau)
        return out

    def pack_scores(self, s):
        """s[h, token] -> score layout."""
        out = np.zeros(self.S)
        for h in range(self.heads):
            for n in range(s.shape[1]):
                out[self.slot(n // self.t, h, n % self.t)] = s[h, n]
        return out

    def unpack_scores(self, slots, ntok):
        return np.array([[slots[self.slot(n // self.t, h, n % self.t)] for n in range(ntok)]
                         for h in range(self.heads)])

    def v_shift(self, k):
        """Right rotation applied to stored V ciphertext k."""
        return (k // self.r_i) * self.r_i * self.H * self.t

    def pack_v(self, V, k):
        out = np.zeros(self.S)
        for e in range(self.E):
            for h in range(self.heads):
                for r in range(self.t):
                    n = ((e + k) % self.E) * self.t + r
                    if n < V.shape[0]:
                        out[self.slot(e, h, r)] = V[n, h, e]
        return np.roll(out, self.v_shift(k))

    def qk_mask(self, c):
        """Keeps copy e = c of the replicated scores of K ciphertext c."""
        m = np.zeros(self.S)
        for h in range(self.H):
            for tau in range(self.t):
                m[self.slot(c % self.E, h, tau)] = 1.0
        return m

    def residue_mask(self, tau):
        m = np.zeros(self.S)
        m[tau::self.t] = 1.0
        return m

    def v_append_mask(self, k, n):
        """Slots of stored V ciphertext k that token n = c*t + tau occupies:
        e = (c - k) mod E at residue tau, moved by the stored rotation."""
        c, tau = n // self.t, n % self.t
        m = np.zeros(self.S)
        for h in range(self.H):
            m[self.slot((c - k) % self.E, h, tau)] = 1.0
        return np.roll(m, self.v_shift(k))

    def v_append_group_mask(self, k, c):
        """Slots of stored V ciphertext k that the t tokens of group c occupy (Sec. 5.4: the
        masked products of the V-cache update, all residues at once): block row e = (c - k) mod E."""
        return sum(self.v_append_mask(k, c * self.t + tau) for tau in range(self.t))

    def pack_k_index(self, K, k):
        """The key index (a re-layout of the K cache, derived from Sec. 5.1's identity: see
        vmm.qk_scores_indexed): ciphertext k = g r_i + j holds at (b, h, tau) element
        K[((b - g r_i) mod E) t + tau, h, (b + j) mod E], i.e. sum_c Rot(mask_c, -g r_i B) Rot(K_c, j B)
        with B = H t slots per copy.  Tokens past the end are zero."""
        g, j = k // self.r_i, k % self.r_i
        out = np.zeros(self.S)
        for b in range(self.E):
            for tau in range(self.t):
                n = ((b - g * self.r_i) % self.E) * self.t + tau
                if n < K.shape[0]:
                    for h in range(self.heads):
                        out[self.slot(b, h, tau)] = K[n, h, (b + j) % self.E]
        return out

    def k_index_append_mask(self, k, n):
        """Slots of index ciphertext k that token n = c*t + tau occupies: copy (c + g r_i) mod E at residue tau."""
        c, tau = n // self.t, n % self.t
        m = np.zeros(self.S)
        for h in range(self.H):
            m[self.slot((c + (k // self.r_i) * self.r_i) % self.E, h, tau)] = 1.0
        return m

    def k_index_append_group_mask(self, k, c):
        return sum(self.k_index_append_mask(k, c * self.t + tau) for tau in range(self.t))

    def k_index_steps(self):
        """Rotation amounts the index needs: the baby steps (of the query, and of a new key at append) and the giant step."""
        s = [j * self.H * self.t for j in range(1, self.r_i)]
        if self.r_o > 1:
            s.append(self.r_i * self.H * self.t)
        return s

    def qk_steps(self):
        return [-(1 << i) for i in range(_log2(self.t))] + \
               [(1 << i) * self.H * self.t for i in range(_log2(self.E))]

    def sv_steps(self):
        s = [j * self.H * self.t for j in range(1, self.r_i)]
        if self.r_o > 1:
            s.append(self.r_i * self.H * self.t)
        return s + [1 << l for l in range(_log2(self.t))]

    def append_steps(self):
        return [-(g * self.r_i * self.H * self.t) for g in range(1, self.r_o)]


# ---- grouped-query attention against a cache that stores every KV head once -------------------------------
@dataclass
class GqaLayout:
    """The paper packs the cache with one K / V head per query head (Sec. 5.3; its Llama-3-8B has H = 32 of
    both).  A model with grouped-query attention has Hkv < H KV heads, each shared by G = H / Hkv query heads;
    repeating every KV head G times fits the paper's layout but stores and appends everything G times.  This
    layout stores each KV head ONCE: the cache is the paper's layout for Hkv heads (`kv`, t_kv = S / (Hkv E)
    tokens per K ciphertext, G times as many as before), the query and the attention output keep the paper's
    layout for H heads (`q`, t = S / (H E)) with head h = hk G + g, and the two meet because

        q.slot(e, hk G + g, tau) == kv.slot(e, hk, g t + tau):

    inside a block of t_kv slots of KV head hk, the G query heads of the group occupy G runs of t residues.
    A query head must meet every token residue j = g' t + tau of its KV head, not only those of its own run,
    so the products run G times, the query moved by the inner rotation (Sec. 5.4) of delta t residues,
    delta = 0 .. G-1: in pass delta the run g' holds query head (g' - delta) mod G.  The scores of a head are
    spread over the G results (token c t_kv + j of head (hk, g) in pass delta = (j // t - g) mod G at slot
    (c, hk, j)); scores V undoes the rotation per pass and sums.  Same number of ciphertext products as the
    replicated layout, 1/G of the cache memory and of the append work, 2 (G - 1) inner rotations per token."""
    S: int
    H: int
    Hkv: int
    E: int
    r_i: int = 0

    def __post_init__(self):
        assert self.H % self.Hkv == 0
        self.G = self.H // self.Hkv
        self.kv = KvLayout(self.S, self.Hkv, self.E, self.r_i)
        self.q = KvLayout(self.S, self.H, self.E)
        self.t = self.q.t
        assert self.kv.t == self.G * self.t
        self.capacity = self.kv.capacity

    def pass_of(self, g, j):
        """The pass in which query head g of a group meets token residue j."""
        return (j // self.t - g) % self.G

    def inner_delta(self, delta):
        """Residues by which the replicated query is moved for pass delta (0 for pass 0)."""
        return delta * self.t

    def pack_scores(self, s):
        """s[h, token] -> the G slot vectors that scores V reads (the layout q K^T writes)."""
        out = [np.zeros(self.S) for _ in range(self.G)]
        tk = self.kv.t
        for h in range(self.H):
            hk, g = divmod(h, self.G)
            for n in range(s.shape[1]):
                c, j = divmod(n, tk)
                out[self.pass_of(g, j)][self.kv.slot(c, hk, j)] = s[h, n]
        return out

    def unpack_scores(self, vecs, ntok):
        tk = self.kv.t
        m = np.zeros((self.H, ntok))
        for h in range(self.H):
            hk, g = divmod(h, self.G)
            for n in range(ntok):
                c, j = divmod(n, tk)
                m[h, n] = vecs[self.pass_of(g, j)][self.kv.slot(c, hk, j)]
        return m

    def qk_steps(self):
        """Replication of the query over its t residues, the inner rotations of the passes, the sum over the dims."""
        s = [-(1 << i) for i in range(_log2(self.t))]
        for delta in range(1, self.G):
            s += self.kv.inner_rotation_steps(self.inner_delta(delta))
        return s + [(1 << i) * self.Hkv * self.kv.t for i in range(_log2(self.E))]

    def sv_steps(self):
        s = [a for a in self.kv.sv_steps() if a % self.kv.t == 0]         # nothing sums over the residues of the cache layout
        for back in range(1, self.G):
            s += self.kv.inner_rotation_steps(self.inner_delta(back))
        return s + [1 << l for l in range(_log2(self.t))]
