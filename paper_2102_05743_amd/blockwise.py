"""Block-by-block processing of sequences that are handed over in pieces (Sec. V-B of the paper: a
block of consecutive steps is one element of the scan).

Protocol, all arithmetic in the library's kernels: every block is reduced to its element
(``hmm_block_element``), the elements give the carries between blocks (``hmm_block_carries``), and each
block is then processed on its own by ``hmm_smooth`` / ``hmm_viterbi`` / ``hmm_max_product`` on its rows
framed by one carry row in front and one lookahead row behind.  This module only allocates the
framed buffers, copies rows into them and slices the results.

Blocks are device tensors [B][T_s][D]; they need not have equal lengths.  ``blocks`` is iterated twice
(elements, then results), so smooth_blocks and max_product_blocks accept any re-iterable, for
instance an object whose ``__iter__`` uploads one block after the other so that only one block is
resident at a time.
"""
from __future__ import annotations

from . import binding as _b


def block_elements(A, blocks, max_product: bool = False):
    """Elements and log-scales of all blocks, stacked: ([S][B][D][D] f32, [S][B] f64)."""
    import torch
    els, lss = [], []
    for ll in blocks:
        if ll.data_ptr() % 16 != 0 or not ll.is_contiguous():
            ll = ll.clone(memory_format=torch.contiguous_format)   # a view into a longer array: the library wants 16-byte alignment
        el, ls = _b.hmm_block_element(A, ll, max_product=max_product)
        els.append(el)
        lss.append(ls)
    return torch.stack(els).contiguous(), torch.stack(lss).contiguous()


def framed_rows(ll, carry_row, lookahead_row):
    """[carry; block; lookahead] for one block: ll[B][T][D], rows [B][D] or None.  Returns the framed
    tensor and the slice of its time axis that holds the block's own steps."""
    import torch
    B, T, D = ll.shape
    lo = 0 if carry_row is None else 1
    n = lo + T + (0 if lookahead_row is None else 1)
    out = torch.empty((B, n, D), dtype=ll.dtype, device=ll.device)
    if carry_row is not None:
        out[:, 0] = carry_row
    out[:, lo:lo + T] = ll
    if lookahead_row is not None:
        out[:, lo + T] = lookahead_row
    return out, slice(lo, lo + T)


def _priors(prior):
    import torch
    return prior, torch.ones_like(prior)


def smooth_blocks(prior, A, blocks, want_filtered: bool = False):
    """Smoothing marginals (and filtered distributions) of every block, as for the whole sequence.
    Returns (list of marginals [B][T_s][D], list of filtered or None, loglik[B] f64)."""
    els, lss = block_elements(A, blocks, max_product=False)
    carry, look, total = _b.hmm_block_carries(prior, A, els, lss, max_product=False)
    S = els.shape[0]
    first, ones = _priors(prior)
    margs, filts = [], []
    for s, ll in enumerate(blocks):
        rows, sl = framed_rows(ll, carry[s] if s > 0 else None, look[s] if s + 1 < S else None)
        m, f, _ = _b.hmm_smooth(first if s == 0 else ones, A, rows, want_filtered=want_filtered)
        margs.append(m[:, sl])
        filts.append(f[:, sl] if want_filtered else None)
    return margs, (filts if want_filtered else None), total


def max_product_blocks(prior, A, blocks):
    """Max-marginals and per-step maximisers of every block, as for the whole sequence.
    Returns (list of max_marginals [B][T_s][D], list of argmax [B][T_s], logprob[B] f64)."""
    els, lss = block_elements(A, blocks, max_product=True)
    carry, look, total = _b.hmm_block_carries(prior, A, els, lss, max_product=True)
    S = els.shape[0]
    first, ones = _priors(prior)
    mms, args = [], []
    for s, ll in enumerate(blocks):
        rows, sl = framed_rows(ll, carry[s] if s > 0 else None, look[s] if s + 1 < S else None)
        mm, am, _ = _b.hmm_max_product(first if s == 0 else ones, A, rows)
        mms.append(mm[:, sl])
        args.append(am[:, sl])
    return mms, args, total


def viterbi_blocks(prior, A, blocks, consistent: bool = True):
    """MAP path of every block.  consistent=True walks the blocks last to first and hands each block the
    first decoded state of the block after it (a one-hot lookahead row), so that the pieces form ONE
    maximising sequence even when several sequences tie; consistent=False uses the lookahead rows of
    hmm_block_carries, which lets all blocks be decoded independently and gives the same path whenever
    the MAP sequence is unique.  Returns (list of paths [B][T_s] int32, logprob[B] f64)."""
    import torch
    els, lss = block_elements(A, blocks, max_product=True)
    carry, look, total = _b.hmm_block_carries(prior, A, els, lss, max_product=True)
    S = els.shape[0]
    first, ones = _priors(prior)
    blocks = list(blocks)
    paths = [None] * S
    nxt = None
    for s in (range(S - 1, -1, -1) if consistent else range(S)):
        if s + 1 == S:
            la = None
        elif consistent:   # the one-hot row of the next block's first decoded state (formatting, no arithmetic)
            la = torch.full_like(look[s], float("-inf"))
            la.scatter_(1, nxt.long().unsqueeze(1), 0.0)
        else:
            la = look[s]
        rows, sl = framed_rows(blocks[s], carry[s] if s > 0 else None, la)
        path, _ = _b.hmm_viterbi(first if s == 0 else ones, A, rows)
        paths[s] = path[:, sl]
        nxt = path[:, sl.start]
    return paths, total
