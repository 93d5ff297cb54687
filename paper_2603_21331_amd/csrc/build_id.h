// The build id of the library this file is compiled into: a hash over the compiler flags and
// the contents of the library's sources, passed in by the build script as RMS_BUILD_ID and kept
// in the binary as a plain string behind a fixed marker, so that the build script can read it
// back from the file and tell a library built from other sources from a current one.
#pragma once

#ifndef RMS_BUILD_ID
#define RMS_BUILD_ID "00000000000000000000000000000000"   /* built by hand, outside the build script */
#endif

#define RMS_DEFINE_BUILD_ID(symbol) \
  extern "C" __attribute__((visibility("default"), used)) const char symbol[] = "RMS_BUILD_ID:" RMS_BUILD_ID
