/* Runs the fp64 C oracle (oracle/ref_attention.c, compiled into this program with
 * -fsanitize=address,undefined) on one case read from a file and writes the results to another.
 * Test infrastructure: tests/test_host_sanitizers.py writes the case, runs this program and compares
 * the results with those of the ordinary build of the oracle.
 *
 * Input file:  int64 header[8] = {G, P, Hq, Hkv, D, n_rows (0: all rows), backward (0/1), 0};
 *              double scale; int32 suffix_lens[G]; float q[T*Hq*D], k_prefix[P*Hkv*D], v_prefix[..],
 *              k_suffix[T*Hkv*D], v_suffix[..]; backward: float d_out[T*Hq*D]; n_rows > 0: int64 rows[n_rows]
 * Output file: forward: double out[n*Hq*D], lse[Hq*n]; backward: double dq[n*Hq*D] and, with all rows,
 *              dk_prefix, dv_prefix [P*Hkv*D], dk_suffix, dv_suffix [T*Hkv*D]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int ref_prefix_shared_attention(const float*, const float*, const float*, const float*, const float*, const int32_t*, int,
                                int64_t, int, int, int, double, const int64_t*, int64_t, double*, double*, int);
int ref_prefix_shared_attention_backward(const float*, const float*, const float*, const float*, const float*,
                                         const float*, const int32_t*, int, int64_t, int, int, int, double,
                                         const int64_t*, int64_t, double*, double*, double*, double*, double*, int);

static void* slurp(FILE* f, size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);
  if (!p || fread(p, 1, bytes, f) != bytes) {
    fprintf(stderr, "oracle_driver: short read\n");
    exit(2);
  }
  return p;
}

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* f = fopen(argv[1], "rb");
  if (!f) return 2;
  int64_t* h = slurp(f, 8 * sizeof(int64_t));
  const int G = (int)h[0], Hq = (int)h[2], Hkv = (int)h[3], D = (int)h[4], backward = (int)h[6];
  const int64_t P = h[1], n_rows = h[5];
  double* scale = slurp(f, sizeof(double));
  int32_t* lens = slurp(f, sizeof(int32_t) * (size_t)G);
  int64_t T = 0;
  for (int g = 0; g < G; ++g) T += lens[g];
  const size_t nq = (size_t)T * Hq * D, nkp = (size_t)P * Hkv * D, nks = (size_t)T * Hkv * D;
  float* q = slurp(f, nq * 4);
  float* kp = slurp(f, nkp * 4);
  float* vp = slurp(f, nkp * 4);
  float* ks = slurp(f, nks * 4);
  float* vs = slurp(f, nks * 4);
  float* d_out = backward ? slurp(f, nq * 4) : NULL;
  int64_t* rows = n_rows ? slurp(f, sizeof(int64_t) * (size_t)n_rows) : NULL;
  fclose(f);
  const int64_t n = n_rows ? n_rows : T;
  const size_t no = (size_t)n * Hq * D;
  FILE* o = fopen(argv[2], "wb");
  if (!o) return 2;
  int rc;
  if (!backward) {
    double* out = malloc(no * 8 + 8);
    double* lse = malloc((size_t)Hq * n * 8 + 8);
    rc = ref_prefix_shared_attention(q, P ? kp : NULL, P ? vp : NULL, ks, vs, lens, G, P, Hq, Hkv, D, *scale, rows, n, out,
                                     lse, 3);
    fwrite(out, 8, no, o);
    fwrite(lse, 8, (size_t)Hq * n, o);
    free(out);
    free(lse);
  } else {
    double* dq = malloc(no * 8 + 8);
    double *dkp = NULL, *dvp = NULL, *dks = NULL, *dvs = NULL;
    if (!rows) {
      dkp = malloc(nkp * 8 + 8);
      dvp = malloc(nkp * 8 + 8);
      dks = malloc(nks * 8 + 8);
      dvs = malloc(nks * 8 + 8);
    }
    rc = ref_prefix_shared_attention_backward(q, P ? kp : NULL, P ? vp : NULL, ks, vs, d_out, lens, G, P, Hq, Hkv, D,
                                              *scale, rows, n, dq, dkp, dvp, dks, dvs, 3);
    fwrite(dq, 8, no, o);
    if (!rows) {
      fwrite(dkp, 8, nkp, o);
      fwrite(dvp, 8, nkp, o);
      fwrite(dks, 8, nks, o);
      fwrite(dvs, 8, nks, o);
    }
    free(dq);
    free(dkp);
    free(dvp);
    free(dks);
    free(dvs);
  }
  fclose(o);
  free(h); free(scale); free(lens); free(q); free(kp); free(vp); free(ks); free(vs); free(d_out); free(rows);
  if (rc < 0) {
    fprintf(stderr, "oracle_driver: the oracle returned %d\n", rc);
    return 3;
  }
  return 0;
}
