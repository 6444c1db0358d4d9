"""CPU oracle of one frontend scheduling round (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; the
product path never does.  It shares no code with the library's host routine: a request here is
its list of token ids and a block of cached prefix is identified by the token prefix itself (a
Python tuple), not by a hash.

What is computed (App. A, Alg. 1; Sec. 7.2 - 7.4; App. B.2):
  * per-GPU block table K_i: which B-token prefix blocks are resident (committed) or promised
    by requests already routed (pending); the match rule reads their union (App. B.2);
  * BlockMatch(K_i, r): tokens covered by the longest run of leading full blocks of the
    request's prefix p_r that K_i holds (Sec. 7.2, block granularity);
  * per request in arrival order: among GPUs with L_i < T take the longest match, ties by the
    smaller load (Alg. 1), remaining ties by the lower GPU index (reading: the paper leaves it
    open); Delta = C_pfx(|p_r| - m) + C_sfx(|s_r|, |p_r|) (Eq. 2); L += Delta; the GPU leaves
    the active set once L >= T; the round stops when no GPU is active or the queue is empty.

Cost model (reading; the paper names the terms of Eq. 2 but prints no formula for them):
  C_pfx(n)    = f_tok*n + f_attn*n(n+1)/2      forward pass over the n uncached prefix tokens
  C_FFN(S)    = f_tok*S                        all linear layers
  C_self(S)   = f_attn*S(S+1)/2                causal self-attention inside the suffix
  C_cross(S,P)= f_attn*S*P                     suffix queries against the prefix's keys
  With f_attn = 0 this is Delta = u*f_tok, u = uncached tokens, the form App. B.2 uses.
"""


def c_pfx(n, f_tok, f_attn):
    return f_tok * n + f_attn * (n * (n + 1) // 2)


def c_sfx(S, P, f_tok, f_attn):
    c_ffn = f_tok * S
    c_self = f_attn * (S * (S + 1) // 2)
    c_cross = f_attn * (S * P)
    return c_ffn + c_self + c_cross


def cost_delta(P, M, S, f_tok, f_attn):
    """Eq. 2."""
    return c_pfx(P - M, f_tok, f_attn) + c_sfx(S, P, f_tok, f_attn)


class BlockTables:
    """K_i for every GPU: committed and pending sets of resident prefix blocks.  A block is the
    tuple of all prompt tokens up to and including it (so equal blocks under different
    histories are different entries, as chained block hashes make them)."""

    def __init__(self, n_gpus, block_tokens):
        self.B = block_tokens
        self.committed = [set() for _ in range(n_gpus)]
        self.pending = [set() for _ in range(n_gpus)]

    def blocks_of(self, prefix_tokens):
        B = self.B
        return [tuple(prefix_tokens[:(j + 1) * B]) for j in range(len(prefix_tokens) // B)]

    def block_match(self, i, prefix_tokens):
        """Tokens of the longest contiguous run of leading blocks present in C_i or P_i."""
        m = 0
        for blk in self.blocks_of(prefix_tokens):
            if blk in self.committed[i] or blk in self.pending[i]:
                m += self.B
            else:
                break
        return m

    def promise(self, i, prefix_tokens):
        for blk in self.blocks_of(prefix_tokens):
            if blk not in self.committed[i]:
                self.pending[i].add(blk)

    def stored(self, i, blocks):
        """Engine event: these blocks are now materialised on GPU i (pending -> committed)."""
        for blk in blocks:
            self.pending[i].discard(blk)
            self.committed[i].add(blk)

    def evicted(self, i, blocks):
        for blk in blocks:
            self.committed[i].discard(blk)


def schedule_round(tables, requests, threshold, f_tok, f_attn, loads=None):
    """One round of Alg. 1, step 1.  requests: list of (prefix_tokens, suffix_len) in arrival
    order.  loads: starting L_i (Alg. 1 starts a round from zero).  Returns a dict with
    assigned[r] (GPU or -1 for requests left in the queue), matched[r], delta[r], loads[i],
    saturated[i] and last_delta[i] (Delta of the last request a GPU took)."""
    n = len(tables.committed)
    L = [0] * n if loads is None else list(loads)
    active = [i for i in range(n) if L[i] < threshold]
    assigned, matched, delta = [], [], []
    last_delta = [None] * n
    for prefix, S in requests:
        if not active:
            assigned.append(-1)
            matched.append(0)
            delta.append(0)
            continue
        m = {i: tables.block_match(i, prefix) for i in active}
        best = max(m.values())
        cands = [i for i in active if m[i] == best]
        low = min(L[i] for i in cands)
        i_star = min(i for i in cands if L[i] == low)
        d = cost_delta(len(prefix), best, S, f_tok, f_attn)
        L[i_star] += d
        tables.promise(i_star, prefix)
        assigned.append(i_star)
        matched.append(best)
        delta.append(d)
        last_delta[i_star] = d
        if L[i_star] >= threshold:
            active.remove(i_star)
    return dict(assigned=assigned, matched=matched, delta=delta, loads=L,
                saturated=[L[i] >= threshold for i in range(n)], last_delta=last_delta)


def tokens_executed(loads, i, tokens, f_tok):
    """App. B.3: the engine reports executed prompt tokens; L_i <- max(0, L_i - tokens * f_tok)."""
    loads = list(loads)
    loads[i] = max(0, loads[i] - tokens * f_tok)
    return loads
