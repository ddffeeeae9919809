// Host-side parts of libdistgrid: error slot, grid descriptor (Sec. 3.2, Sec. 4.1), weight counts.
#include "dg_internal.h"
#include <cmath>
#include <cstring>

namespace dg {
static thread_local char g_error[256] = "";
void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
}
}  // namespace dg

extern "C" const char *dg_last_error(void) { return dg::g_error; }

extern "C" double dg_growth_factor(uint32_t N_min, uint32_t N_max, uint32_t L)
{
    if (L < 2 || N_min == 0) return 1.0;
    return std::exp(std::log((double)N_max / (double)N_min) / (double)(L - 1));
}

extern "C" int dg_grid_desc_init(dg_grid_desc *desc, uint32_t L, uint32_t F, uint32_t log2_T,
                                 uint32_t N_min, double growth, const double extent[3])
{
    DG_REQUIRE(desc && extent, DG_ERR_ARG, "dg_grid_desc_init: null pointer");
    DG_REQUIRE(L >= 1 && N_min >= 1 && growth >= 1.0, DG_ERR_ARG, "dg_grid_desc_init: L, N_min >= 1 and growth >= 1 required");
    DG_REQUIRE(extent[0] > 0 && extent[1] > 0 && extent[2] > 0, DG_ERR_ARG, "dg_grid_desc_init: box extents must be positive");
    DG_REQUIRE(L <= DG_MAX_LEVELS && F == 2 && log2_T <= 24, DG_ERR_UNSUPPORTED,
               "dg_grid_desc_init: need L <= 16, F == 2, log2_T <= 24 (got %u, %u, %u)", L, F, log2_T);
    std::memset(desc, 0, sizeof *desc);
    desc->n_levels = L;
    desc->n_features = F;
    desc->log2_T = log2_T;
    const double longest = std::fmax(extent[0], std::fmax(extent[1], extent[2]));
    const uint64_t T = 1ull << log2_T;
    uint64_t cursor = 0;
    double n = (double)N_min;   // N_min * growth^l, built by pow() per level below
    for (uint32_t l = 0; l < L; ++l) {
        n = std::floor((double)N_min * std::pow(growth, (double)l) + 1e-6);
        DG_REQUIRE(n < 1048576.0, DG_ERR_UNSUPPORTED, "dg_grid_desc_init: level %u resolution too large", l);
        desc->n_voxels[l] = (uint32_t)n;
        uint64_t vertices = 1;
        for (int a = 0; a < 3; ++a) {
            const double cells = extent[a] / longest * n;
            uint32_t r = (uint32_t)std::ceil(cells);
            desc->res[l][a] = r ? r : 1u;
            desc->scale[l][a] = (float)cells;
            vertices *= (uint64_t)desc->res[l][a] + 1u;
        }
        desc->dense[l] = vertices <= T ? 1u : 0u;
        desc->offset[l] = (uint32_t)cursor;
        cursor += desc->dense[l] ? (vertices + 7u) / 8u * 8u : T;
        DG_REQUIRE(cursor <= 0xffffffffull, DG_ERR_UNSUPPORTED, "dg_grid_desc_init: table exceeds 2^32 entries");
    }
    desc->offset[L] = (uint32_t)cursor;
    desc->n_entries = (uint32_t)cursor;
    return DG_OK;
}

extern "C" size_t dg_mlp_weight_count(const dg_mlp_desc *m)
{
    if (!m) return 0;
    size_t c = (size_t)m->n_hidden_d * m->n_feat + (size_t)m->n_geo * m->n_hidden_d +
               (size_t)m->n_hidden_c * (m->n_geo + m->n_dir) + 3u * (size_t)m->n_hidden_c;
    if (m->n_layers_c == 2) c += (size_t)m->n_hidden_c * m->n_hidden_c;
    c += (size_t)m->n_hidden_c * m->n_app;      // the appearance columns of the first colour layer, packed last
    return c;
}
