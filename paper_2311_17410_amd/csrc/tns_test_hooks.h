// Hooks for the library's own tests: accepted in tns_config.flags but not part of the public header.
#pragma once

// Test of the fused kernel's bounded wait: the tile tickets start at 1, so the first tile's predecessor
// never reports.  Every kernel still ends (after the bound, about two seconds); tns_run_status then
// reports the time-out and the dense outputs are not valid.
#define TNS_TEST_FLAG_LOST_TILE 64
