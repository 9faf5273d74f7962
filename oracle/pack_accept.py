"""CPU oracle: tree packing and the greedy accept walk.  TEST INFRASTRUCTURE ONLY.

Neither step is spelled out in the paper (a tree is verified "in a single
forward pass", Sec. 1; a draft path is "accepted" prefix by prefix, Sec. 3.1
below Eq. "cum_prob"); both are written here from their plain definitions.
"""
from __future__ import annotations

MAX_NODES = 128  # ancestor masks are 128 bits: two 64-bit words per node


def pack(cu_nodes, parent, prefix_len):
    """Per node: depth, position id, owning sequence, ancestor-or-self bitmask.

    depth(root) = 0, depth(i) = depth(parent(i)) + 1
    position(i) = prefix_len[b] + depth(i)
    mask(i)     = mask(parent(i)) | (1 << i)      (local node ids, 128 bits,
                  returned as (low word, high word))
    """
    N = int(cu_nodes[-1])
    depth = [0] * N
    position = [0] * N
    node_seq = [0] * N
    mask = [(0, 0)] * N
    for b in range(len(cu_nodes) - 1):
        base = int(cu_nodes[b])
        n_b = int(cu_nodes[b + 1]) - base
        if n_b > MAX_NODES:
            raise ValueError("tree exceeds 128 nodes")
        full = [0] * n_b
        for i in range(n_b):
            p = int(parent[base + i])
            if i == 0:
                if p != -1:
                    raise ValueError("node 0 must be the root")
                full[i] = 1
                depth[base] = 0
            else:
                if not (0 <= p < i):
                    raise ValueError("parents must precede children")
                full[i] = full[p] | (1 << i)
                depth[base + i] = depth[base + p] + 1
            position[base + i] = int(prefix_len[b]) + depth[base + i]
            node_seq[base + i] = b
            mask[base + i] = (full[i] & 0xFFFFFFFFFFFFFFFF, full[i] >> 64)
    return depth, position, node_seq, mask


def accept(cu_nodes, parent, token, target_next, max_depth):
    """Greedy longest accepted path per sequence.

    Start at the root.  From the current node cur, the target model's own next
    token is target_next[cur]; move to the child of cur whose drafted token
    equals it (smallest node id if several siblings carry the same token);
    stop when there is none.  accept_len counts accepted draft nodes (the root
    is not a draft), accept_path lists the visited local node ids (root first,
    padded with -1 to max_depth + 1), bonus_token = target_next at the last
    node reached.
    """
    B = len(cu_nodes) - 1
    accept_len = [0] * B
    bonus = [0] * B
    paths = [[-1] * (max_depth + 1) for _ in range(B)]
    for b in range(B):
        base = int(cu_nodes[b])
        n_b = int(cu_nodes[b + 1]) - base
        cur = 0
        path = [0]
        while len(path) <= max_depth:
            want = int(target_next[base + cur])
            nxt = -1
            for j in range(cur + 1, n_b):
                if int(parent[base + j]) == cur and int(token[base + j]) == want:
                    nxt = j
                    break
            if nxt < 0:
                break
            cur = nxt
            path.append(cur)
        accept_len[b] = len(path) - 1
        bonus[b] = int(target_next[base + cur])
        for d, v in enumerate(path):
            paths[b][d] = v
    return accept_len, paths, bonus


def accept_by_path_enumeration(cu_nodes, parent, token, target_next, max_depth):
    """Independent statement of the same result: enumerate every root-to-leaf
    path, measure how long a prefix of it the target agrees with, keep the
    longest (first in leaf order on ties).  Used only to pin ``accept``."""
    B = len(cu_nodes) - 1
    lens = [0] * B
    ends = [0] * B
    for b in range(B):
        base = int(cu_nodes[b])
        n_b = int(cu_nodes[b + 1]) - base
        has_child = [False] * n_b
        for j in range(1, n_b):
            has_child[int(parent[base + j])] = True
        best_len, best_end = 0, 0
        for leaf in range(n_b):
            if has_child[leaf]:
                continue
            chain = []
            v = leaf
            while v >= 0:
                chain.append(v)
                v = int(parent[base + v])
            chain.reverse()
            matched = 0
            for d in range(1, len(chain)):
                if d > max_depth:
                    break
                prev, node = chain[d - 1], chain[d]
                if int(token[base + node]) != int(target_next[base + prev]):
                    break
                # a smaller-numbered sibling carrying the same token wins the tie
                dup = any(int(parent[base + s]) == prev and
                          int(token[base + s]) == int(token[base + node])
                          for s in range(prev + 1, node))
                if dup:
                    break
                matched = d
            if matched > best_len:
                best_len, best_end = matched, chain[matched]
        lens[b] = best_len
        ends[b] = best_end
    return lens, ends


def commit(cu_nodes, accept_len, accept_path, k_tree, v_tree, k_cache, v_cache, block_table,
           prefix_len, max_depth):
    """Makes the tokens a verify step produced part of their sequences.

    A step yields, per sequence, the root and the accept_len accepted draft
    nodes (the path tree_accept walked; "accepted" prefix by prefix, Sec. 3.1
    below Eq. "cum_prob").  Node accept_path[b][i] sits at depth i, so its
    position id is prefix_len[b] + i: its K/V row goes to that token position
    of sequence b's paged cache (block block_table[b][pos // block_size], slot
    pos % block_size), and the prefix grows to prefix_len[b] + accept_len[b] + 1.

    Plain layout on this side: k_cache, v_cache are [num_blocks][Hkv][block_size][D]
    numpy arrays, modified in place; k_tree, v_tree are [N][Hkv][D].
    Returns (new_prefix_len, status); status[b] is 0, -3 (no room in the block
    table: nothing is written for b and its length stays) or -2 (a path that is
    not a path of the tree's size: same treatment).
    """
    B = len(cu_nodes) - 1
    block_size = k_cache.shape[2]
    max_blocks = block_table.shape[1]
    new_len = [int(x) for x in prefix_len]
    status = [0] * B
    for b in range(B):
        base = int(cu_nodes[b])
        n_b = int(cu_nodes[b + 1]) - base
        a = int(accept_len[b])
        nodes = [int(accept_path[b][i]) for i in range(max(0, min(a, max_depth)) + 1)]
        if a < 0 or a > max_depth or any(not (0 <= v < n_b) for v in nodes):
            status[b] = -2
            continue
        start = int(prefix_len[b])
        if start < 0 or start + a + 1 > max_blocks * block_size:
            status[b] = -3
            continue
        blocks = [int(block_table[b][(start + i) // block_size]) for i in range(a + 1)]
        if any(not (0 <= blk < k_cache.shape[0]) for blk in blocks):
            status[b] = -2
            continue
        for i, v in enumerate(nodes):
            pos = start + i
            k_cache[blocks[i], :, pos % block_size, :] = k_tree[base + v]
            v_cache[blocks[i], :, pos % block_size, :] = v_tree[base + v]
        new_len[b] = start + a + 1
    return new_len, status
