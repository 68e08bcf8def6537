// Reads sharding-planner problems from stdin, runs amsp_plan_sharding (csrc/amsp_planner.cpp, compiled into
// this program with -fsanitize=address,undefined by tests/test_sanitizers_cpu.py) and prints the plans with
// their doubles as hexadecimal floats, so that the test can compare them exactly with the Python oracle.
//   problem:  phi layers micro_batches bucket_bytes R N memory activation tmp nmods nrows
//             nmods doubles
//             nrows lines "op p0 p1 bytes bytes_per_s"
#include <stdio.h>

#include <vector>

#include "amsp.h"

int main() {
    amsp_plan_problem pb;
    unsigned nmods, nrows;
    while (scanf("%lf %u %u %lf %u %u %lf %lf %lf %u %u", &pb.phi, &pb.layers, &pb.micro_batches, &pb.bucket_bytes,
                 &pb.gpus_per_node, &pb.nodes, &pb.gpu_memory_bytes, &pb.activation_bytes, &pb.tmp_bytes, &nmods,
                 &nrows) == 11) {
        std::vector<double> mods(nmods);
        for (double &x : mods)
            if (scanf("%lf", &x) != 1) return 2;
        std::vector<amsp_bw_sample> table(nrows);
        for (amsp_bw_sample &r : table)
            if (scanf("%u %u %u %lf %lf", &r.op, &r.p0, &r.p1, &r.bytes, &r.bytes_per_s) != 5) return 2;
        pb.modules_per_layer = nmods;
        pb.module_params = mods.data();
        amsp_plan best;
        uint32_t count = 0;
        const int rc = amsp_plan_sharding(&pb, table.data(), nrows, &best, &count);
        if (rc != AMSP_OK) {
            printf("status %d\n", rc);
            continue;
        }
        printf("status 0 %u %u %u %u %u %u %a %a %a %a %a %a %u\n", best.sp0, best.sp1, best.sg0, best.sg1, best.sos0,
               best.sos1, best.t_p, best.t_g, best.t_os0, best.t_os1, best.t_comm, best.d_modelstate, count);
    }
    return 0;
}
