// Host-only check of the binary band kernel's geometry: prints one line for the shape given on the command line
// (n h w c_in c_out k stride pad groups), or "no" when the layer cannot be created.
#include <cstdio>
#include <cstdlib>

#include "bin_shape.h"

int main(int argc, char** argv) {
    if (argc != 10) return 2;
    rrm_shape s{};
    s.kind = RRM_CONV;
    s.n = atoi(argv[1]); s.h = atoi(argv[2]); s.w = atoi(argv[3]); s.c_in = atoi(argv[4]); s.c_out = atoi(argv[5]);
    s.kh = s.kw = atoi(argv[6]); s.stride = atoi(argv[7]); s.pad = atoi(argv[8]); s.groups = atoi(argv[9]);
    rrm::BinGeom g{};
    if (!rrm::bin_choose_shape(s, g)) {
        printf("no\n");
        return 0;
    }
    printf("ho=%d wo=%d R=%d nbands=%d bth=%d btw=%d lds=%zu wlds=%d vec4=%d fused=%d pitch=%d nslab=%d\n", g.ho, g.wo, g.band_rows,
           g.nbands, g.bth_in, g.btw_in, g.band_rows > 0 ? rrm::bin_band_lds_bytes(g, g.band_rows) : (size_t)0, g.wlds, g.vec4,
           g.fused_ok, g.pitch, g.nslab);
    return 0;
}
