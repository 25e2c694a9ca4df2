/* Test infrastructure: runs the oracle's primitives and a whole small flow in a build with
 * -fsanitize=address,undefined (make -C oracle asan), so that an out-of-bounds access, a signed
 * overflow or a misaligned load in the oracle fails a CPU test instead of silently shaping the
 * expected values. It only calls the oracle and copies bytes; it holds none of the method's
 * arithmetic.
 *
 *   sanitize_driver rq                       reads "a M s" triples from stdin, prints rq and sat8(rq)
 *   sanitize_driver flow BLOB X B OUT        x u8 [B,3,H,W] from file X -> OUT: z, codes, x after
 *                                            decode, containers + sizes, x after container decode
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "iodf_oracle.h"

static void* slurp(const char* path, size_t* n) {
    FILE* f = fopen(path, "rb");
    if (!f) { perror(path); exit(2); }
    fseek(f, 0, SEEK_END);
    long sz = ftell(f);
    fseek(f, 0, SEEK_SET);
    void* p = malloc(sz > 0 ? (size_t)sz : 1);
    if (sz > 0 && fread(p, 1, (size_t)sz, f) != (size_t)sz) { perror("read"); exit(2); }
    fclose(f);
    *n = (size_t)sz;
    return p;
}

int main(int argc, char** argv) {
    if (argc >= 2 && !strcmp(argv[1], "rq")) {
        long a, M, s;
        while (scanf("%ld %ld %ld", &a, &M, &s) == 3) {
            const int64_t r = orc_rq((int32_t)a, (int32_t)M, (int)s);
            printf("%lld %d\n", (long long)r, (int)orc_sat8(r));
        }
        return 0;
    }
    if (argc == 6 && !strcmp(argv[1], "flow")) {
        size_t nb, nx;
        void* blob = slurp(argv[2], &nb);
        uint8_t* x = (uint8_t*)slurp(argv[3], &nx);
        const int B = atoi(argv[4]);
        orc_model* m = NULL;
        if (orc_model_load(blob, nb, &m) != 0) { fprintf(stderr, "bad blob\n"); return 3; }
        const int64_t d = orc_model_d(m), dc = orc_model_d_codes(m), cap = orc_codec_max_words(m);
        if ((size_t)(B * d) != nx) { fprintf(stderr, "image file does not hold %d images\n", B); return 3; }
        int32_t* z = (int32_t*)malloc(sizeof(int32_t) * (size_t)(B * d));
        int8_t* codes = (int8_t*)malloc((size_t)(B * dc) + 1);
        uint8_t* x2 = (uint8_t*)malloc((size_t)(B * d));
        uint8_t* x3 = (uint8_t*)malloc((size_t)(B * d));
        uint32_t* cont = (uint32_t*)calloc((size_t)(B * cap), sizeof(uint32_t));
        uint32_t* sizes = (uint32_t*)calloc((size_t)B, sizeof(uint32_t));
        int64_t errs = 0, clamped = 0, derr = 0;
        if (orc_forward(m, x, B, z, dc ? codes : NULL) != 0) return 4;
        if (orc_inverse(m, z, B, x2, &errs) != 0) return 4;
        if (orc_encode(m, x, B, cont, cap, sizes, &clamped) != 0) return 4;
        if (orc_decode(m, cont, cap, B, x3, &derr) != 0) return 4;
        FILE* f = fopen(argv[5], "wb");
        if (!f) { perror(argv[5]); return 2; }
        fwrite(z, sizeof(int32_t), (size_t)(B * d), f);
        fwrite(codes, 1, (size_t)(B * dc), f);
        fwrite(x2, 1, (size_t)(B * d), f);
        fwrite(cont, sizeof(uint32_t), (size_t)(B * cap), f);
        fwrite(sizes, sizeof(uint32_t), (size_t)B, f);
        fwrite(x3, 1, (size_t)(B * d), f);
        fclose(f);
        printf("d %lld d_codes %lld cap %lld range_errors %lld clamped %lld decode_errors %lld\n", (long long)d,
               (long long)dc, (long long)cap, (long long)errs, (long long)clamped, (long long)derr);
        orc_model_free(m);
        free(blob); free(x); free(z); free(codes); free(x2); free(x3); free(cont); free(sizes);
        return 0;
    }
    fprintf(stderr, "usage: sanitize_driver rq | flow BLOB X B OUT\n");
    return 2;
}
