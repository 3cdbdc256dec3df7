/*
 * Driver that runs the C oracle's entry points under AddressSanitizer / UndefinedBehaviorSanitizer on the host.
 * TEST INFRASTRUCTURE: compiled by tests/test_oracle_sanitizers.py together with oracle/dense_oracle.c
 * (gcc -fsanitize=address,undefined) and run in a subprocess.
 *
 * Input file (little endian):  int64 V, E_out, E_in, n_targets, k, direction, seed, then
 *   int64 rowptr_out[V+1], int32 col_out[E_out], (if E_in >= 0: int64 rowptr_in[V+1], int32 col_in[E_in]),
 *   int32 targets[n_targets], int32 fanouts[k].
 * Output file: int64 rc, N, E, then int64 node_id_offsets[k+2], int32 node_ids[N], int64 nbr_offsets[N - n_0 + 1],
 *   int32 nbrs[E], int32 repr_map[E], then the gathered rows of a small int32 table whose row r is (r, 2r, 3r).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_dense_sample(int64_t V, const int64_t* rowptr_out, const int32_t* col_out, const int64_t* rowptr_in,
                     const int32_t* col_in, int32_t direction, const int32_t* targets, int32_t n_targets, int32_t k,
                     const int32_t* fanouts, uint64_t seed, int64_t cap_nodes, int64_t cap_nbrs,
                     int64_t* node_id_offsets_out, int32_t* node_ids_out, int64_t* nbr_offsets_out, int32_t* nbrs_out,
                     int32_t* repr_map_out, int64_t* counts);
void orc_dense_gather(const uint8_t* table, int64_t ld_bytes, int64_t row_bytes, const int32_t* node_ids, int64_t n,
                      uint8_t* H0);

static void* must_read(FILE* f, size_t bytes)
{
    void* p = malloc(bytes ? bytes : 1);
    if (!p || (bytes && fread(p, 1, bytes, f) != bytes)) { fprintf(stderr, "short input\n"); exit(3); }
    return p;
}

int main(int argc, char** argv)
{
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    int64_t* hdr = (int64_t*)must_read(f, 7 * sizeof(int64_t));
    const int64_t V = hdr[0], E_out = hdr[1], E_in = hdr[2], n_targets = hdr[3], k = hdr[4], direction = hdr[5];
    const uint64_t seed = (uint64_t)hdr[6];
    int64_t* rp_out = (int64_t*)must_read(f, sizeof(int64_t) * (size_t)(V + 1));
    int32_t* col_out = (int32_t*)must_read(f, sizeof(int32_t) * (size_t)E_out);
    int64_t* rp_in = NULL;
    int32_t* col_in = NULL;
    if (E_in >= 0) {
        rp_in = (int64_t*)must_read(f, sizeof(int64_t) * (size_t)(V + 1));
        col_in = (int32_t*)must_read(f, sizeof(int32_t) * (size_t)E_in);
    }
    int32_t* targets = (int32_t*)must_read(f, sizeof(int32_t) * (size_t)n_targets);
    int32_t* fanouts = (int32_t*)must_read(f, sizeof(int32_t) * (size_t)k);
    fclose(f);

    /* exact capacities: an overrun of one element is an overrun of the allocation */
    const int mult = direction == 2 ? 2 : 1;
    int64_t level = n_targets, cap_nodes = n_targets, cap_nbrs = 0;
    for (int64_t h = 0; h < k; ++h) {
        level = level * fanouts[h] * mult;
        cap_nbrs += level;
        cap_nodes += level < V ? level : V;
    }
    if (cap_nodes > V) cap_nodes = V;
    int64_t* node_id_offsets = (int64_t*)malloc(sizeof(int64_t) * (size_t)(k + 2));
    int32_t* node_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap_nodes ? cap_nodes : 1));
    int64_t* nbr_offsets = (int64_t*)malloc(sizeof(int64_t) * (size_t)(cap_nodes + 1));
    int32_t* nbrs = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap_nbrs ? cap_nbrs : 1));
    int32_t* repr_map = (int32_t*)malloc(sizeof(int32_t) * (size_t)(cap_nbrs ? cap_nbrs : 1));
    int64_t counts[2] = { 0, 0 };
    const int64_t rc = orc_dense_sample(V, rp_out, col_out, rp_in, col_in, (int32_t)direction, targets, (int32_t)n_targets,
                                        (int32_t)k, fanouts, seed, cap_nodes, cap_nbrs, node_id_offsets, node_ids,
                                        nbr_offsets, nbrs, repr_map, counts);
    FILE* o = fopen(argv[2], "wb");
    if (!o) return 2;
    const int64_t head[3] = { rc, counts[0], counts[1] };
    fwrite(head, sizeof(int64_t), 3, o);
    if (rc == 0) {
        const int64_t N = counts[0], E = counts[1], with_nbrs = N - node_id_offsets[1];
        fwrite(node_id_offsets, sizeof(int64_t), (size_t)(k + 2), o);
        fwrite(node_ids, sizeof(int32_t), (size_t)N, o);
        fwrite(nbr_offsets, sizeof(int64_t), (size_t)(with_nbrs + 1), o);
        fwrite(nbrs, sizeof(int32_t), (size_t)E, o);
        fwrite(repr_map, sizeof(int32_t), (size_t)E, o);
        int32_t* table = (int32_t*)malloc(sizeof(int32_t) * 3 * (size_t)V);
        for (int64_t r = 0; r < V; ++r) { table[3 * r] = (int32_t)r; table[3 * r + 1] = (int32_t)(2 * r); table[3 * r + 2] = (int32_t)(3 * r); }
        int32_t* h0 = (int32_t*)malloc(sizeof(int32_t) * 3 * (size_t)(N ? N : 1));
        orc_dense_gather((const uint8_t*)table, 12, 12, node_ids, N, (uint8_t*)h0);
        fwrite(h0, sizeof(int32_t), (size_t)(3 * N), o);
        free(table); free(h0);
    }
    fclose(o);
    free(hdr); free(rp_out); free(col_out); free(rp_in); free(col_in); free(targets); free(fanouts);
    free(node_id_offsets); free(node_ids); free(nbr_offsets); free(nbrs); free(repr_map);
    return 0;
}
