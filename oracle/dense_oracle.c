/*
 * dense_oracle.c -- plain, slow CPU oracle for DENSE mini-batch construction (single-threaded; one loop, the
 * per-node one-hop sample, carries an OpenMP pragma that a second build of the same file switches on).  TEST INFRASTRUCTURE ONLY: it is called by the tests, by the smoke
 * check and by the benchmark's cpu_baseline leg; the product path never links,
 * loads or calls it, and it shares no code with the HIP kernels.
 *
 * What it follows (MariusGNN paper, Section 4.1):
 *   - Algorithm 1 "Multi-hop Neighborhood Sampling" in the paper's own order: k rounds,
 *     each round one-hop-samples Delta_i, stacks the result IN FRONT of nbrs /
 *     nbr_offsets, computes Delta_{i-1} = unique(Delta_i_nbrs) \ node_ids and stacks it
 *     in front of node_ids / node_id_offsets.
 *   - Section 4.2, first paragraph: repr_map[j] = index in H^0 (= position in node_ids)
 *     of nbrs[j]; H^0 row r = base representation of node_ids[r].
 *
 * Readings of points the paper leaves open (they make the result unique, so that a
 * second implementation can be compared bit for bit):
 *   - one-hop sampling (Section 4.1: "more than f neighbours -> only f are sampled,
 *     fewer -> all are returned") is uniform WITHOUT replacement by Floyd's subset
 *     algorithm (Bentley & Floyd, CACM 30(9), 1987) over adjacency positions; random
 *     words come from Philox4x32-10 (Salmon et al., SC'11) with
 *         counter = (s >> 2, node id, hop, direction bit),  key = (seed lo, seed hi),
 *     word s & 3 for Floyd step s, reduced to [0, j] by a 32x32 multiply-high;
 *     hop = distance from the targets (targets are hop 0);
 *   - neighbours are stored in Floyd insertion order when deg > f and in adjacency order
 *     otherwise;
 *   - each Delta_{i-1} is in ascending node id; Delta_k keeps the caller's order;
 *   - fanouts are ordered away from the targets (Section 7.1): hop h uses fanouts[h],
 *     i.e. Algorithm 1's round i = k - h;
 *   - both offset arrays carry an end sentinel (node_id_offsets has k+2 entries,
 *     nbr_offsets has (#nodes with neighbours)+1), which Algorithm 2 needs on the
 *     last layer;
 *   - direction 2 (incoming and outgoing, Section 7.1): a node's segment is its
 *     out-sample followed by its in-sample, each drawn with the hop's fanout.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- Philox4x32-10 */

static void philox_round(uint32_t c[4], const uint32_t k[2])
{
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k[0];
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k[1];
    const uint32_t n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

/* out = Philox4x32-10(counter, key): ten rounds, the key advanced by the two Weyl
 * constants before every round but the first. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c[4] = { ctr[0], ctr[1], ctr[2], ctr[3] };
    uint32_t k[2] = { key[0], key[1] };
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k[0] += 0x9E3779B9u; k[1] += 0xBB67AE85u; }
        philox_round(c, k);
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* ---------------------------------------------------------------- one-hop sample */

/* Uniform f-subset of adjacency positions [0, deg) by Floyd's algorithm, in insertion
 * order.  picks must hold f entries.  Requires deg > f >= 1. */
void orc_floyd_positions(int64_t deg, int32_t f, uint64_t seed, uint32_t node, uint32_t hop,
                         uint32_t dirbit, int64_t* picks)
{
    const uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    for (int32_t s = 0; s < f; ++s) {
        const int64_t j = deg - f + s;
        const uint32_t ctr[4] = { (uint32_t)(s >> 2), node, hop, dirbit };
        uint32_t w[4];
        orc_philox4x32_10(ctr, key, w);
        const uint32_t r = w[s & 3];
        const int64_t t = (int64_t)(((uint64_t)r * (uint64_t)(j + 1)) >> 32);   /* in [0, j] */
        int present = 0;
        for (int32_t q = 0; q < s; ++q) if (picks[q] == t) present = 1;
        picks[s] = present ? j : t;
    }
}

/* Sampled neighbours of node v along one direction; returns how many were written. */
int32_t orc_onehop_dir(const int64_t* rowptr, const int32_t* col, int32_t v, int32_t f,
                       uint64_t seed, uint32_t hop, uint32_t dirbit, int32_t* out)
{
    const int64_t base = rowptr[v];
    const int64_t deg = rowptr[v + 1] - base;
    if (deg <= f) {
        for (int64_t p = 0; p < deg; ++p) out[p] = col[base + p];
        return (int32_t)deg;
    }
    int64_t* picks = (int64_t*)malloc(sizeof(int64_t) * (size_t)f);
    orc_floyd_positions(deg, f, seed, (uint32_t)v, hop, dirbit, picks);
    for (int32_t s = 0; s < f; ++s) out[s] = col[base + picks[s]];
    free(picks);
    return f;
}

/* direction: 0 = out-edges (rowptr_out/col_out), 1 = in-edges, 2 = out then in. */
int32_t orc_onehop(const int64_t* rowptr_out, const int32_t* col_out,
                   const int64_t* rowptr_in, const int32_t* col_in, int32_t direction,
                   int32_t v, int32_t f, uint64_t seed, uint32_t hop, int32_t* out)
{
    int32_t c = 0;
    if (direction == 0 || direction == 2)
        c += orc_onehop_dir(rowptr_out, col_out, v, f, seed, hop, 0u, out + c);
    if (direction == 1 || direction == 2)
        c += orc_onehop_dir(rowptr_in, col_in, v, f, seed, hop, 1u, out + c);
    return c;
}

/* ---------------------------------------------------------------- Algorithm 1 */

static int cmp_i32(const void* a, const void* b)
{
    const int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

/* cat(front, back) into a fresh array */
static int32_t* cat_i32(const int32_t* front, int64_t nf, const int32_t* back, int64_t nb)
{
    int32_t* r = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nf + nb + 1));
    if (nf > 0) memcpy(r, front, sizeof(int32_t) * (size_t)nf);       /* an empty part may come as a null pointer */
    if (nb > 0) memcpy(r + nf, back, sizeof(int32_t) * (size_t)nb);
    return r;
}

/* cat(front, back + shift) into a fresh array */
static int64_t* cat_i64_shift(const int64_t* front, int64_t nf, const int64_t* back, int64_t nb, int64_t shift)
{
    int64_t* r = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nf + nb + 1));
    if (nf > 0) memcpy(r, front, sizeof(int64_t) * (size_t)nf);
    for (int64_t i = 0; i < nb; ++i) r[nf + i] = back[i] + shift;
    return r;
}

/*
 * Multi-hop sampling into DENSE + repr_map.
 *
 * Outputs (caller-allocated):
 *   node_id_offsets int64[k+2]   start of Delta_0..Delta_k in node_ids, then N
 *   node_ids        int32[cap_nodes]
 *   nbr_offsets     int64[cap_nodes+1]  entry q = start in nbrs of the node at position
 *                                       node_id_offsets[1]+q; last entry = E
 *   nbrs, repr_map  int32[cap_nbrs]
 *   counts          int64[2] = {N, E}
 * Returns 0, or -1 bad argument (id out of range, duplicate target, k < 1, fanout < 1),
 * -2 capacity exceeded.
 */
int orc_dense_sample(int64_t V,
                     const int64_t* rowptr_out, const int32_t* col_out,
                     const int64_t* rowptr_in, const int32_t* col_in, int32_t direction,
                     const int32_t* targets, int32_t n_targets,
                     int32_t k, const int32_t* fanouts, uint64_t seed,
                     int64_t cap_nodes, int64_t cap_nbrs,
                     int64_t* node_id_offsets_out, int32_t* node_ids_out,
                     int64_t* nbr_offsets_out, int32_t* nbrs_out, int32_t* repr_map_out,
                     int64_t* counts)
{
    if (k < 1 || n_targets < 0 || direction < 0 || direction > 2) return -1;
    for (int32_t h = 0; h < k; ++h) if (fanouts[h] < 1) return -1;
    const int ndir = (direction == 2) ? 2 : 1;

    uint8_t* in_node_ids = (uint8_t*)calloc((size_t)V, 1);      /* membership of node_ids */
    for (int32_t i = 0; i < n_targets; ++i) {
        const int32_t t = targets[i];
        if (t < 0 || t >= V || in_node_ids[t]) { free(in_node_ids); return -1; }
        in_node_ids[t] = 1;
    }

    /* Line 1-2: node_id_offsets = [0]; node_ids = targets; nbr_offsets = []; nbrs = []; Delta_k = targets */
    int64_t n_off = 1;
    int64_t* node_id_offsets = (int64_t*)malloc(sizeof(int64_t) * 2); node_id_offsets[0] = 0;
    int64_t n_ids = n_targets;
    int32_t* node_ids = cat_i32(targets, n_targets, NULL, 0);
    int64_t n_nbr_off = 0;
    int64_t* nbr_offsets = (int64_t*)malloc(sizeof(int64_t));
    int64_t n_nbrs = 0;
    int32_t* nbrs = (int32_t*)malloc(sizeof(int32_t));
    int64_t n_delta = n_targets;
    int32_t* delta = cat_i32(targets, n_targets, NULL, 0);
    int rc = 0;

    for (int32_t i = k; i >= 1; --i) {
        const int32_t hop = k - i;                 /* distance of Delta_i from the targets */
        const int32_t f = fanouts[hop];

        /* Line 4: Delta_i_nbrs, Delta_i_offsets = oneHopSample(Delta_i, fanouts[i]).
         * The nodes' samples are independent of each other (Section 4.1 runs them on several threads): every node
         * samples into a stretch of its own, long enough for the largest sample; the stretches are then packed in
         * node order.  Built with -fopenmp the first loop runs on all cores; without it the pragma is ignored.
         * The result is the same either way. */
        const int64_t stretch = (int64_t)f * ndir;
        int32_t* sampled = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_delta * stretch + 1));
        int32_t* sampled_count = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_delta + 1));
#pragma omp parallel for schedule(dynamic, 256)
        for (int64_t q = 0; q < n_delta; ++q)
            sampled_count[q] = orc_onehop(rowptr_out, col_out, rowptr_in, col_in, direction,
                                          delta[q], f, seed, (uint32_t)hop, sampled + q * stretch);
        int32_t* d_nbrs = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_delta * stretch + 1));
        int64_t* d_offsets = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_delta + 1));
        int64_t n_d_nbrs = 0;
        for (int64_t q = 0; q < n_delta; ++q) {
            d_offsets[q] = n_d_nbrs;
            if (sampled_count[q] > 0)
                memcpy(d_nbrs + n_d_nbrs, sampled + q * stretch, sizeof(int32_t) * (size_t)sampled_count[q]);
            n_d_nbrs += sampled_count[q];
        }
        free(sampled); free(sampled_count);

        /* Line 5: nbr_offsets = cat(Delta_i_offsets, nbr_offsets + len(Delta_i_nbrs)) */
        int64_t* new_nbr_offsets = cat_i64_shift(d_offsets, n_delta, nbr_offsets, n_nbr_off, n_d_nbrs);
        free(nbr_offsets); nbr_offsets = new_nbr_offsets; n_nbr_off += n_delta;
        /* Line 6: nbrs = cat(Delta_i_nbrs, nbrs) */
        int32_t* new_nbrs = cat_i32(d_nbrs, n_d_nbrs, nbrs, n_nbrs);
        free(nbrs); nbrs = new_nbrs; n_nbrs += n_d_nbrs;

        /* Line 7: Delta_{i-1} = unique nodes of Delta_i_nbrs that are not in node_ids, ascending */
        int32_t* cand = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_d_nbrs + 1));
        int64_t n_cand = 0;
        for (int64_t j = 0; j < n_d_nbrs; ++j)
            if (!in_node_ids[d_nbrs[j]]) cand[n_cand++] = d_nbrs[j];
        qsort(cand, (size_t)n_cand, sizeof(int32_t), cmp_i32);
        int64_t n_next = 0;
        for (int64_t j = 0; j < n_cand; ++j)
            if (j == 0 || cand[j] != cand[j - 1]) cand[n_next++] = cand[j];

        /* Line 8: node_id_offsets = cat([0], node_id_offsets + len(Delta_{i-1})) */
        const int64_t zero = 0;
        int64_t* new_off = cat_i64_shift(&zero, 1, node_id_offsets, n_off, n_next);
        free(node_id_offsets); node_id_offsets = new_off; n_off += 1;
        /* Line 9: node_ids = cat(Delta_{i-1}, node_ids) */
        int32_t* new_ids = cat_i32(cand, n_next, node_ids, n_ids);
        free(node_ids); node_ids = new_ids; n_ids += n_next;
        for (int64_t j = 0; j < n_next; ++j) in_node_ids[cand[j]] = 1;

        free(delta); delta = cand; n_delta = n_next;
        free(d_nbrs); free(d_offsets);
    }

    if (n_ids > cap_nodes || n_nbrs > cap_nbrs) rc = -2;
    if (rc == 0) {
        for (int64_t j = 0; j < n_off; ++j) node_id_offsets_out[j] = node_id_offsets[j];
        node_id_offsets_out[n_off] = n_ids;                                   /* end sentinel */
        memcpy(node_ids_out, node_ids, sizeof(int32_t) * (size_t)n_ids);
        for (int64_t j = 0; j < n_nbr_off; ++j) nbr_offsets_out[j] = nbr_offsets[j];
        nbr_offsets_out[n_nbr_off] = n_nbrs;                                  /* end sentinel */
        memcpy(nbrs_out, nbrs, sizeof(int32_t) * (size_t)n_nbrs);

        /* repr_map: position in node_ids of every entry of nbrs (Section 4.2) */
        int32_t* position = (int32_t*)malloc(sizeof(int32_t) * (size_t)V);
        for (int64_t r = 0; r < n_ids; ++r) position[node_ids[r]] = (int32_t)r;
        for (int64_t j = 0; j < n_nbrs; ++j) repr_map_out[j] = position[nbrs[j]];
        free(position);
        counts[0] = n_ids; counts[1] = n_nbrs;
    }
    free(in_node_ids); free(node_id_offsets); free(node_ids); free(nbr_offsets); free(nbrs); free(delta);
    return rc;
}

/* ---------------------------------------------------------------- H^0 gather */

/* H0[r, :] = table[node_ids[r], :], rows of row_bytes bytes, table rows ld_bytes apart. */
void orc_dense_gather(const uint8_t* table, int64_t ld_bytes, int64_t row_bytes,
                      const int32_t* node_ids, int64_t n, uint8_t* H0)
{
    for (int64_t r = 0; r < n; ++r)
        memcpy(H0 + r * row_bytes, table + (int64_t)node_ids[r] * ld_bytes, (size_t)row_bytes);
}
