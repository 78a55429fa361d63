"""Brute-force enumeration of the chunk list of a ragged tensor list.

TEST INFRASTRUCTURE ONLY.  The paper clips "per parameter tensor" (Sec. 4.2,
Eq. 3); a GPU implementation has to cut each tensor into pieces of bounded
size.  The only facts that matter are integer ones: every element of every
tensor belongs to exactly one piece, pieces never span two tensors, and pieces
are cut at multiples of the chunk size counted from the tensor's own first
element.  This walks the elements tensor by tensor and writes those pieces
down, one Python step per piece, with no closed-form index arithmetic.
"""


def enumerate_chunks(numels, chunk_elems):
    """Return (chunks, chunk_begin) where chunks is a list of
    (tensor_index, first_element, length) in list order and chunk_begin[i] is
    the position of tensor i's first chunk (chunk_begin[n] = total)."""
    chunks = []
    chunk_begin = []
    for i, numel in enumerate(numels):
        chunk_begin.append(len(chunks))
        first = 0
        remaining = int(numel)
        while remaining > 0:
            length = chunk_elems if remaining > chunk_elems else remaining
            chunks.append((i, first, length))
            first += length
            remaining -= length
    chunk_begin.append(len(chunks))
    return chunks, chunk_begin
