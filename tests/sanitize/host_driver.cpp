// Sanitizer run of the library's host-side table code (csrc/nm_tables.cpp: descriptor validation,
// the chord / Algorithm 3 / Algorithm 2 table builder, table objects' error paths), compiled for the
// host only with -fsanitize=address,undefined by tests/test_sanitizers.py.  Output arrays have
// exactly the documented size.  No GPU call is reached: every nm_build_tables call below fails
// validation first.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "nm.h"

#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED %s (line %d): %s\n", #cond, __LINE__, nm_last_error()); return 1; } } while (0)

int main()
{
    static const float range[7][2] = {{-8, 8}, {-16, 0}, {1, 64}, {1e-3f, 64}, {-8, 8}, {0.25f, 64}, {-3, 5}};
    for (int f = 0; f < 7; ++f)
        for (int nseg : {1, 2, 3, 37, 128, 1000, NM_MAX_SEGMENTS})
            for (int flags : {0, (int)NM_TABLE_CLAMP_INPUT, (int)NM_TABLE_BIAS_CORRECT, (int)NM_TABLE_MERGE, (int)(NM_TABLE_MERGE | NM_TABLE_BIAS_CORRECT)}) {
                nm_table_desc d{};
                d.func = f; d.lo = range[f][0]; d.hi = range[f][1]; d.nseg = nseg; d.flags = flags; d.e_th = 1e-4f; d.dk_th = 0.02f;
                float* k = static_cast<float*>(std::malloc(sizeof(float) * nseg));
                float* b = static_cast<float*>(std::malloc(sizeof(float) * nseg));
                float inv_w = 0; int32_t nd = 0;
                EXPECT(nm_table_build_host(&d, k, b, &inv_w, &nd) == NM_OK);
                EXPECT(nd >= 1 && nd <= nseg && inv_w > 0);
                EXPECT(nm_table_build_host(&d, k, b, &inv_w, nullptr) == NM_OK);
                std::free(k); std::free(b);
            }
    // descriptors that must be refused, for the host builder and for the table objects alike
    nm_table_desc bad[] = {{NM_FUNC_EXP, 0, 0, 8, 0, 0, 0}, {NM_FUNC_EXP, 0, 1, 0, 0, 0, 0}, {99, 0, 1, 8, 0, 0, 0},
                           {NM_FUNC_RECIP, 0, 1, 8, 0, 0, 0}, {NM_FUNC_RSQRT, -1, 1, 8, 0, 0, 0},
                           {NM_FUNC_EXP, 0, 1, NM_MAX_SEGMENTS + 1, 0, 0, 0}, {NM_FUNC_GELU, -1, 1, 8, NM_TABLE_MERGE, 0, -1.0f}};
    float k[8], b[8], iw;
    for (const nm_table_desc& d : bad) {
        EXPECT(nm_table_build_host(&d, k, b, &iw, nullptr) != NM_OK);
        nm_tables* t = nullptr;
        EXPECT(nm_build_tables(&d, 1, nullptr, &t) != NM_OK && t == nullptr);
    }
    nm_tables* t = nullptr;
    EXPECT(nm_build_tables(nullptr, 1, nullptr, &t) == NM_ERR_INVALID_ARG);
    EXPECT(nm_build_tables(bad, 0, nullptr, &t) == NM_ERR_INVALID_ARG);
    EXPECT(nm_build_tables(bad, NM_MAX_TABLES + 1, nullptr, &t) != NM_OK);
    EXPECT(nm_tables_count(nullptr) == 0);
    EXPECT(nm_tables_get(nullptr, 0, nullptr, nullptr, nullptr, nullptr) != NM_OK);
    nm_tables_destroy(nullptr);
    EXPECT(nm_version() >= 1000);
    std::printf("SANITIZE_OK\n");
    return 0;
}
