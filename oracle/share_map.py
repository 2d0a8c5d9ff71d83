"""Oracle of the structural part of the strategy search (Algorithm 1), test infrastructure only.

The paper ranks all layer pairs by the Euclidean distance of their KV representations,
largest first, and walks the ranking: a pair joins the strategy if the model with the
candidate strategy still resembles the original (the similarity test, which needs a model
and is therefore a caller-supplied predicate here), until C layers are shared.  In a pair
the layer nearer the output takes the cache of the layer nearer the input (Sec. 3.1.2,
"Sharing Strategy Searching").

Readings the paper leaves open (they are part of this oracle's definition):
  * ties in the ranking keep (i, j) lexicographic order;
  * strategies stay depth one: a pair (i < j) is passed over, without a similarity test
    and without counting, when j already receives a cache, when j already donates one, or
    when i already receives one; a donor may serve several recipients;
  * KV-store slots number the layers that keep their own cache in increasing layer order.
"""
import math

OK, TARGET_UNREACHED = 0, -4


def build_share_map(dist, L, C, ascending=False, accept=None):
    """Return (status, share_map, slot_of_layer, n_slots, n_shared)."""
    pairs = []
    for i in range(L):
        for j in range(i + 1, L):
            v = float(dist[i][j])
            if math.isnan(v):
                raise ValueError("NaN distance")
            pairs.append((v, i, j))
    pairs.sort(key=lambda t: (t[0] if ascending else -t[0], t[1], t[2]))
    share = list(range(L))
    donors = set()
    shared = 0
    for _, i, j in pairs:
        if shared == C:
            break
        if share[j] != j or j in donors or share[i] != i:
            continue
        cand = list(share)
        cand[j] = i
        if accept is not None and not accept(cand):
            continue
        share = cand
        donors.add(i)
        shared += 1
    slot, nxt = [0] * L, 0
    for l in range(L):
        if share[l] == l:
            slot[l] = nxt
            nxt += 1
    for l in range(L):
        if share[l] != l:
            slot[l] = slot[share[l]]
    return (OK if shared == C else TARGET_UNREACHED), share, slot, nxt, shared
